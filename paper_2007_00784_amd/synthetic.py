"""Seeded synthetic workloads: layer shape tables and input tensors.

This module holds no K-FAC arithmetic.  It only describes the layer sets the
benchmarks and tests run on (shapes of ResNet-50 for 224x224 inputs and of the
CIFAR ResNet-32, the networks of the paper's Sec. VI-B) and draws the input
tensors -- activations, output gradients, weight gradients -- from a
counter-based generator, so that every consumer sees identical bytes whatever
the chunking or thread count.

Generator: value e of a stream is a pure function of (key, e).  The 64-bit key
is a hash chain over (seed, workload id, layer index, tensor kind, update
index); uniforms come from a SplitMix64-style finaliser of key + counter and
are turned into normals with the Box-Muller transform in float64, two normals
per counter pair, then cast to float32.
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
import os

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)

KIND_X, KIND_G, KIND_GRADW, KIND_CHSCALE = 1, 2, 3, 4


def _mix(z):
    """SplitMix64 finaliser on a uint64 array (wrapping arithmetic)."""
    z = (z ^ (z >> np.uint64(30))) * _C1
    z = (z ^ (z >> np.uint64(27))) * _C2
    return z ^ (z >> np.uint64(31))


def make_key(*parts):
    """Hash chain over integer parts -> uint64 stream key."""
    with np.errstate(over="ignore"):
        k = np.array([0x243F6A8885A308D3], dtype=np.uint64)
        for p in parts:
            k = _mix((k ^ _mix(np.array([int(p) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64) + _GOLD)) + _GOLD)
    return np.uint64(k[0])


def _uniform(key, idx):
    """Open-interval uniforms in (0,1) for uint64 counters idx."""
    with np.errstate(over="ignore"):
        z = _mix(key + (idx + np.uint64(1)) * _GOLD)
    return ((z >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _normal_chunk(key, start, stop):
    """Standard normals for element indices [start, stop) of stream key (float64)."""
    p0, p1 = start // 2, (stop + 1) // 2
    pair = np.arange(p0, p1, dtype=np.uint64)
    u1 = _uniform(key, pair * np.uint64(2))
    u2 = _uniform(key, pair * np.uint64(2) + np.uint64(1))
    r = np.sqrt(-2.0 * np.log(u1))
    th = (2.0 * np.pi) * u2
    z = np.empty((p1 - p0) * 2, dtype=np.float64)
    z[0::2] = r * np.cos(th)
    z[1::2] = r * np.sin(th)
    return z[start - 2 * p0: stop - 2 * p0]


def normal(key, n, sigma=1.0, relu=False, chunk=1 << 20, workers=None):
    """n float32 values: sigma * N(0,1), optionally max(0, .) before scaling."""
    out = np.empty(n, dtype=np.float32)
    bounds = [(s, min(s + chunk, n)) for s in range(0, n, chunk)]

    def work(b):
        z = _normal_chunk(key, b[0], b[1])
        if relu:
            np.maximum(z, 0.0, out=z)
        out[b[0]:b[1]] = (z * sigma).astype(np.float32)

    if workers is None:
        workers = min(16, os.cpu_count() or 1)
    if len(bounds) > 1 and workers > 1:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(work, bounds))
    else:
        for b in bounds:
            work(b)
    return out


def uniform(key, n):
    return _uniform(key, np.arange(n, dtype=np.uint64))


def to_bf16_bits(a):
    """Round float32 -> bfloat16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# layer descriptors
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Layer:
    name: str
    c_in: int
    c_out: int
    k: int          # square kernel; 1 for FC
    stride: int
    pad: int
    h_in: int       # square input map; 1 for FC
    fc: bool = False

    @property
    def h_out(self):
        return (self.h_in + 2 * self.pad - self.k) // self.stride + 1

    @property
    def T(self):
        return self.h_out * self.h_out

    @property
    def d_a(self):          # with the bias column
        return self.c_in * self.k * self.k + 1

    @property
    def d_g(self):
        return self.c_out

    def rows(self, n):
        return n * self.T

    @property
    def needs_unfold(self):
        """False when the patch matrix is the activation tensor itself (1x1, stride 1, no pad; FC)."""
        return not (self.k == 1 and self.stride == 1 and self.pad == 0)


BOTTLENECK_BLOCKS = {50: (3, 4, 6, 3), 101: (3, 4, 23, 3), 152: (3, 8, 36, 3)}


def resnet50_layers(depth=50):
    """Convs + FC of a bottleneck ResNet (depth 50: 53 convs; 101: 104; 152: 155) on 224x224 inputs; stride of
    a down-sampling block on its 3x3."""
    L = [Layer("stem", 3, 64, 7, 2, 3, 224)]
    h, c_prev = 56, 64
    for si, (width, blocks) in enumerate(zip((64, 128, 256, 512), BOTTLENECK_BLOCKS[depth])):
        c_out = 4 * width
        for b in range(blocks):
            s = 2 if (b == 0 and si > 0) else 1
            h_in = h
            pre = "s%db%d" % (si + 1, b)
            L.append(Layer(pre + ".reduce", c_prev, width, 1, 1, 0, h_in))
            L.append(Layer(pre + ".conv3", width, width, 3, s, 1, h_in))
            h = h_in // s
            L.append(Layer(pre + ".expand", width, c_out, 1, 1, 0, h))
            if b == 0:
                L.append(Layer(pre + ".proj", c_prev, c_out, 1, s, 0, h_in))
            c_prev = c_out
    L.append(Layer("fc", 2048, 1000, 1, 1, 0, 1, fc=True))
    return L


def resnet32_cifar_layers():
    """CIFAR ResNet-32 on 32x32 inputs: stem, 3 stages x 5 blocks x 2 convs, 1x1 projection shortcuts, FC."""
    L = [Layer("stem", 3, 16, 3, 1, 1, 32)]
    h, c_prev = 32, 16
    for si, width in enumerate([16, 32, 64]):
        for b in range(5):
            s = 2 if (b == 0 and si > 0) else 1
            pre = "s%db%d" % (si + 1, b)
            L.append(Layer(pre + ".conv1", c_prev, width, 3, s, 1, h))
            if s == 2:
                L.append(Layer(pre + ".short", c_prev, width, 1, 2, 0, h))
            h //= s
            L.append(Layer(pre + ".conv2", width, width, 3, 1, 1, h))
            c_prev = width
    L.append(Layer("fc", 64, 10, 1, 1, 0, 1, fc=True))
    return L


@dataclass(frozen=True)
class Workload:
    wid: int                 # enters the RNG key
    name: str
    layers: tuple
    batch: int
    sigma_g: float
    damping: float
    decay: float = 0.95
    seed: int = 0
    bf16: bool = False
    ill_conditioned: bool = False
    sigma_gradw: float = 1e-2


def workload(name):
    """The five benchmark configurations and two deeper layer sets (shapes and distributions only)."""
    if name == "single_conv":
        return Workload(1, name, (Layer("conv", 16, 16, 3, 1, 1, 8),), 32, 1e-3, 1e-3)
    if name == "resnet32_cifar":
        return Workload(2, name, tuple(resnet32_cifar_layers()), 128, 1e-3, 3e-3)
    if name == "resnet50":
        return Workload(3, name, tuple(resnet50_layers()), 32, 1e-4, 1e-3)
    if name == "largest_factor":
        return Workload(4, name, (Layer("l4conv3", 512, 512, 3, 1, 1, 7),), 64, 1e-4, 1e-3, ill_conditioned=True)
    if name == "resnet50_bf16":
        return Workload(5, name, tuple(resnet50_layers()), 64, 1e-4, 1e-3, seed=1, bf16=True)
    # the deeper models of the paper's scaling study (Sec. VI-C, Table V): same layer shapes, more of them
    if name == "resnet101":
        return Workload(6, name, tuple(resnet50_layers(101)), 32, 1e-4, 1e-3)
    if name == "resnet152":
        return Workload(7, name, tuple(resnet50_layers(152)), 32, 1e-4, 1e-3)
    # a stack of Linear layers only (the other layer kind the method handles, Sec. V): samples are [R][d] rows, no
    # unfold anywhere, factors of rank <= batch
    if name == "mlp":
        widths = (2048, 2048, 2048, 1000)
        layers = tuple(Layer("fc%d" % i, widths[i], widths[i + 1], 1, 1, 0, 1, fc=True) for i in range(len(widths) - 1))
        return Workload(8, name, layers, 256, 1e-3, 1e-3)
    raise KeyError(name)


def layer_inputs(wl, li, update=0, batch=None, want=("x", "g", "gradw")):
    """float32 master tensors of layer li of workload wl for factor update `update`.

    x     [N, C, H, W]   ReLU(N(0,1))  (FC: [N, C]); channel c scaled by 10**u_c, u_c ~ U[-3,1],
                         when the workload is ill-conditioned
    g     [N, C_out, Ho, Wo]  N(0, sigma_g^2)  (FC: [N, C_out])
    gradw [d_G, d_A]     N(0, sigma_gradw^2), last column = bias gradient
    """
    lay = wl.layers[li]
    n = wl.batch if batch is None else batch
    out = {}
    if "x" in want:
        shape = (n, lay.c_in) if lay.fc else (n, lay.c_in, lay.h_in, lay.h_in)
        x = normal(make_key(wl.seed, wl.wid, li, KIND_X, update), int(np.prod(shape)), relu=True).reshape(shape)
        if wl.ill_conditioned:
            u = uniform(make_key(wl.seed, wl.wid, li, KIND_CHSCALE, 0), lay.c_in)
            sc = (10.0 ** (-3.0 + 4.0 * u)).astype(np.float32)
            x = x * (sc.reshape(1, -1) if lay.fc else sc.reshape(1, -1, 1, 1))
        out["x"] = np.ascontiguousarray(x, dtype=np.float32)
    if "g" in want:
        shape = (n, lay.c_out) if lay.fc else (n, lay.c_out, lay.h_out, lay.h_out)
        out["g"] = normal(make_key(wl.seed, wl.wid, li, KIND_G, update), int(np.prod(shape)),
                          sigma=wl.sigma_g).reshape(shape)
    if "gradw" in want:
        out["gradw"] = normal(make_key(wl.seed, wl.wid, li, KIND_GRADW, update), lay.d_g * lay.d_a,
                              sigma=wl.sigma_gradw).reshape(lay.d_g, lay.d_a)
    return out
