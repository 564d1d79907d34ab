"""Seeded synthetic layer-size chains and checkpoint masks.

This module only produces inputs: it holds none of the method's arithmetic and
is the one module that both the GPU path's callers and the CPU oracle's tests
draw from, so both see the very same arrays.

Random values come from a counter-based generator: the SplitMix64 output
function applied to a counter built from (seed, stream, chain, position), so
any element can be regenerated on its own and the arrays do not depend on
generation order or chunking.

Arrays are position-major ("structure of arrays"): ``d[k, c]`` is the size of
layer output k of chain c, shape ``(n+1, batch)``, int64; masks have the same
shape, uint8.  ``chain_major(x)`` gives the ``(batch, n+1)`` copy.

The paper's workloads are the layer-output sizes of CNN chains (VGG-19,
AlexNet; Section 5.1); ``vgg19_chain`` rebuilds the VGG-19 one from the layer
list given there, the ResNet-shaped chains and the random chains stand in for
larger models.
"""
import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    """SplitMix64 output function on a uint64 array (wrapping arithmetic)."""
    z = (z + _GOLD).astype(np.uint64)
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def random_u64(seed, stream, n_pos, batch, chain0=0, chains=None):
    """uint64 array (n_pos, batch): element (k, c) depends only on
    (seed, stream, chain0 + c, k); with `chains` (an array of `batch` chain
    numbers) on (seed, stream, chains[c], k) instead."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([(int(seed) << 8) ^ int(stream)], dtype=np.uint64))
        ids = np.arange(batch, dtype=np.uint64) + np.uint64(chain0) if chains is None \
            else np.asarray(chains, dtype=np.uint64)
        chain = ids << np.uint64(20)
        pos = np.arange(n_pos, dtype=np.uint64)
        ctr = chain[None, :] | pos[:, None]
        return _mix(_mix(ctr ^ key))


def uniform_aligned_chains(seed, n_layers, batch, lo_units, hi_units, unit=4096, chain0=0, chains=None):
    """Sizes unit * U{lo_units..hi_units}, shape (n_layers+1, batch)."""
    r = random_u64(seed, 0, n_layers + 1, batch, chain0, chains)
    span = np.uint64(hi_units - lo_units + 1)
    return ((r % span).astype(np.int64) + np.int64(lo_units)) * np.int64(unit)


def log_uniform_chains(seed, n_layers, batch, lo_log2=16.0, hi_log2=28.0, chain0=0):
    """Sizes floor(2^(lo + (hi-lo) u)), u uniform in [0,1): unaligned bytes."""
    r = random_u64(seed, 0, n_layers + 1, batch, chain0)
    u = (r >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    d = np.floor(np.exp2(lo_log2 + (hi_log2 - lo_log2) * u)).astype(np.int64)
    return np.maximum(d, 1)


def bernoulli_masks(seed, n_layers, batch, p=0.25, chain0=0, chains=None):
    """Checkpoint masks: interior positions set with probability p, both ends
    forced to 1.  Shape (n_layers+1, batch), uint8."""
    r = random_u64(seed, 1, n_layers + 1, batch, chain0, chains)
    thresh = np.uint64(min(int(p * 2.0 ** 64), 2 ** 64 - 1))
    m = (r < thresh).astype(np.uint8)
    m[0, :] = 1
    m[n_layers, :] = 1
    return m


def chain_major(x):
    """(n+1, batch) -> contiguous (batch, n+1)."""
    return np.ascontiguousarray(x.T)


def ragged_batch(seed, lengths, lo_units=256, hi_units=32768, unit=4096, p=0.25, named=()):
    """Chains of different n in one flat array: (d, mask, offsets).  Chain c has lengths[c] layers,
    sizes unit * U{lo_units..hi_units} drawn as chain c of `uniform_aligned_chains` with its own n,
    and a `bernoulli_masks` mask; d[offsets[c]:offsets[c+1]] are its sizes d_0..d_n.  `named` is a
    list of (index, column) pairs: those chains take the given sizes instead (their lengths must
    agree), e.g. the chains built from the paper's layer lists."""
    lengths = np.asarray(lengths, dtype=np.int64)
    offsets = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(lengths + 1, out=offsets[1:])
    d = np.empty(int(offsets[-1]), dtype=np.int64)
    m = np.empty(int(offsets[-1]), dtype=np.uint8)
    for n in np.unique(lengths):
        idx = np.nonzero(lengths == n)[0]          # all chains of this length at once
        at = offsets[idx][None, :] + np.arange(int(n) + 1, dtype=np.int64)[:, None]
        d[at] = uniform_aligned_chains(seed, int(n), len(idx), lo_units, hi_units, unit, chains=idx)
        m[at] = bernoulli_masks(seed, int(n), len(idx), p, chains=idx)
    for c, col in named:
        col = np.asarray(col, dtype=np.int64).reshape(-1)
        assert col.size == lengths[c] + 1
        d[offsets[c]:offsets[c + 1]] = col
    return d, m, offsets


def _column(sizes):
    return np.asarray(sizes, dtype=np.int64).reshape(-1, 1)


def resnet152_chain(batch_size=64, bytes_per=4):
    """n = 152: input, stem, 3/8/36/3 bottleneck blocks of three layers with
    widths (C/4, C/4, C) at 56/28/14/7 pixels, classifier."""
    B = batch_size * bytes_per
    sizes = [B * 3 * 224 * 224, B * 64 * 112 * 112]
    for hw, c, blocks in ((56, 256, 3), (28, 512, 8), (14, 1024, 36), (7, 2048, 3)):
        for _ in range(blocks):
            sizes += [B * (c // 4) * hw * hw, B * (c // 4) * hw * hw, B * c * hw * hw]
    sizes.append(B * 1000)
    assert len(sizes) == 153
    return _column(sizes)


def resnet1001_chain(batch_size=32, bytes_per=4):
    """n = 1001: input, stem, 3 stages of 111 bottleneck blocks with widths
    (w, w, 4w), w = 16/32/64 at 32/16/8 pixels, classifier."""
    B = batch_size * bytes_per
    sizes = [B * 3 * 32 * 32, B * 16 * 32 * 32]
    for hw, w in ((32, 16), (16, 32), (8, 64)):
        for _ in range(111):
            sizes += [B * w * hw * hw, B * w * hw * hw, B * 4 * w * hw * hw]
    sizes.append(B * 10)
    assert len(sizes) == 1002
    return _column(sizes)


def vgg19_chain(batch_size=128, bytes_per=4):
    """n = 24: the 16 convolution, 5 max-pooling and 3 fully connected layers
    of VGG-19 on a 224x224 crop (Section 5.1), fp32 outputs."""
    B = batch_size * bytes_per
    sizes = [B * 3 * 224 * 224]
    hw = 224
    for c, convs in ((64, 2), (128, 2), (256, 4), (512, 4), (512, 4)):
        sizes += [B * c * hw * hw] * convs
        hw //= 2
        sizes.append(B * c * hw * hw)
    sizes += [B * 4096, B * 4096, B * 1000]
    assert len(sizes) == 25
    return _column(sizes)


def alexnet_chain(batch_size=128, bytes_per=4):
    """n = 15: AlexNet in the paper's extended specs (Section 5.4, "Standalone
    Max-Pooling Layers"; Section 5.1.3 counts AdaptiveAvgPool2d, Flatten and
    Dropout as layers): 5 convolutions, 3 standalone max-poolings, the average
    pooling, flatten, two dropouts and 3 fully connected layers on a 224x224
    crop, fp32 outputs."""
    B = batch_size * bytes_per
    shapes = [3 * 224 * 224,
              64 * 55 * 55, 64 * 27 * 27, 192 * 27 * 27, 192 * 13 * 13,      # conv, pool, conv, pool
              384 * 13 * 13, 256 * 13 * 13, 256 * 13 * 13, 256 * 6 * 6,      # conv x3, pool
              256 * 6 * 6, 9216, 9216, 4096, 4096, 4096, 1000]               # avgpool, flatten, dropout, fc, dropout, fc, fc
    assert len(shapes) == 16
    return _column([B * s for s in shapes])


# The five benchmark configurations ------------------------------------------------

def config1():
    """Single chain, n = 12, 1-64 MiB in 4 KiB multiples, seed 0."""
    return uniform_aligned_chains(0, 12, 1, 256, 16384)


def config2():
    return resnet152_chain()


def config3(batch=65536):
    """n = 64, log-uniform 64 KiB..256 MiB, seed 1; masks p = 0.25."""
    return log_uniform_chains(1, 64, batch), bernoulli_masks(1, 64, batch)


def config4():
    return resnet1001_chain()


def config5_single(n_layers=4096):
    """Single chain, 1-128 MiB in 4 KiB multiples, seed 2."""
    return uniform_aligned_chains(2, n_layers, 1, 256, 32768)


def config5_batch(batch=1048576, n_layers=256, chain0=0):
    """Same distribution, seed 2 (stream of chains offset by one so that chain
    0 is not the single chain above); masks p = 0.25."""
    d = uniform_aligned_chains(2, n_layers, batch, 256, 32768, chain0=chain0 + 1)
    m = bernoulli_masks(2, n_layers, batch, chain0=chain0 + 1)
    return d, m
