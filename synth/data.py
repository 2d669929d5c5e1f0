"""Seeded synthetic weights, images and schemes for the five benchmark workloads.

The paper scores schemes on CIFAR-10 with trained networks; neither is
available, so inputs of the same shape stand in for them: 32x32x3 fp32 images
drawn N(0,1), 10 classes, He-normal weights.  "Folded BN" weights are produced
directly by the recipe: a He-normal filter bank scaled per output channel by a
positive gain g = gamma / sqrt(var + eps) with a bias beta - mean * g, the four
BN statistics drawn from narrow distributions.  That is a value distribution
for the inputs, not a step of the scored method (the method receives folded
tensors).

One numpy ``Generator(PCG64(seed))`` with ``seed = 14090 + workload index`` is
consumed in a fixed order: per node (weights, then BN statistics or classifier
bias), then images, then schemes.

Workloads 7-10 repeat 2, 3, 5 and 6 (own seeds) with a *centred classifier*:
with random weights the pooled feature vector is dominated by a component
common to all images, so the plain recipe makes the FP32 model predict one
class for every image and no scheme ever changes a prediction.  For these
workloads the classifier bias is a stored constant (``centred_bias.json``)
equal to minus the classifier's response to the mean pooled feature of the
workload's first 64 images, so that the FP32 predictions spread over the
classes and low-bit layers flip a visible fraction of them.  The constants are
written by ``oracle/write_centred_bias.py`` (CPU oracle only); this module just
reads them.
"""
from __future__ import annotations

import json
import os

import numpy as np

from . import graphs as G

BITS_ALPHABET = (32, 16, 8, 6, 4, 2)
BN_EPS = np.float32(1e-5)


def weight_shape(node):
    """[cout][k] row-major; k = (cin/groups)*kh*kw in (ci, ky, kx) order."""
    if node["kind"] == G.KIND_DEPTHWISE:
        return (node["cout"], node["kh"] * node["kw"])
    if node["kind"] == G.KIND_FC:
        return (node["cout"], node["cin"])
    return (node["cout"], node["cin"] * node["kh"] * node["kw"])


def make_model(nodes, rng, trivial_bn=False):
    """Returns (weights, biases): per node fp32 arrays [cout][k] and [cout]."""
    weights, biases = [], []
    for node in nodes:
        cout, k = weight_shape(node)
        w = (rng.standard_normal((cout, k)) * np.sqrt(2.0 / k)).astype(np.float32)
        if node["kind"] == G.KIND_FC:
            b = (rng.standard_normal(cout) * 0.1).astype(np.float32)
        else:
            gamma = rng.uniform(0.8, 1.2, cout).astype(np.float32)
            beta = (rng.standard_normal(cout) * 0.1).astype(np.float32)
            mean = (rng.standard_normal(cout) * 0.1).astype(np.float32)
            var = rng.uniform(0.8, 1.2, cout).astype(np.float32)
            if trivial_bn:
                gamma[:], beta[:], mean[:], var[:] = 1.0, 0.0, 0.0, 1.0
                g = gamma
            else:
                g = (gamma / np.sqrt(var + BN_EPS)).astype(np.float32)
            w = (w * g[:, None]).astype(np.float32)
            b = (beta - mean * g).astype(np.float32)
        weights.append(np.ascontiguousarray(w))
        biases.append(np.ascontiguousarray(b))
    return weights, biases


def make_images(n, rng, hin=32):
    """fp32 [n][hin][hin][3] (NHWC), N(0,1)."""
    return rng.standard_normal((n, hin, hin, 3)).astype(np.float32)


CENTRED_OF = {7: 2, 8: 3, 9: 5, 10: 6}  # workload -> the workload whose structure it repeats
CENTRE_IMAGES = 64                       # images the stored classifier bias was formed on
_BIAS_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "centred_bias.json")


def centred_bias(index):
    """Stored classifier bias (fp32 [classes]) of a centred workload; KeyError if it was never written."""
    with open(_BIAS_FILE) as f:
        table = json.load(f)
    return np.array([float.fromhex(v) for v in table[str(index)]], dtype=np.float32)


def _choice_schemes(rng, s, L, alphabet):
    return rng.choice(np.array(alphabet, dtype=np.uint8), size=(s, L)).astype(np.uint8)


def make_workload(index, n_images=None, n_schemes=None, centred=True):
    """The benchmark workloads, numbered as the five configurations.

    0: ResNet-8, 256 images, 1 scheme from {32,8,4}
    1: ResNet-20, 1024 images, 1 scheme from {32,16,8,4}
    2: ResNet-20 greedy step, 1024 images, 40 single-layer schemes (layer i at 8 or 4)
    3: MobileNetV2-32, 512 images, 16 schemes with 10 random layers at 4 bits
    4: ResNet-20 coordinate-descent sweep, 10000 images, 64 schemes from all six widths
    5: PlainConvNet20 sensitivity sweep, 256 images, 42 single-layer schemes (layer i at 8 or 4)
    6: HeavyEarlyResNet20 sensitivity sweep, 256 images, 40 single-layer schemes
  (5 and 6 are the paper's two variant models with the candidate batch of its per-layer
  sensitivity table; they are not among the five benchmark configurations.)
    7, 8, 9, 10: workloads 2, 3, 5, 6 again with their own seeds and a centred classifier (module
  docstring); ``centred=False`` leaves the drawn classifier bias in place (used by the script that
  writes the stored constants).
    ``n_images`` / ``n_schemes`` shrink a workload for tests; the draw order is
    unchanged so weights do not depend on them.
    """
    rng = np.random.Generator(np.random.PCG64(14090 + index))
    seed_index, index = index, CENTRED_OF.get(index, index)
    if index == 0:
        nodes, n, name = G.resnet_cifar(1), 256, "resnet8_n256_s1"
    elif index in (1, 2, 4):
        nodes = G.resnet_cifar(3)
        n = {1: 1024, 2: 1024, 4: 10000}[index]
        name = {1: "resnet20_n1024_s1", 2: "resnet20_greedy_step_n1024_s40",
                4: "resnet20_cd_sweep_n10000_s64"}[index]
    elif index == 3:
        nodes, n, name = G.mobilenetv2_32(), 512, "mobilenetv2_32_n512_s16"
    elif index == 5:
        nodes, n, name = G.plain_convnet20(), 256, "plainconvnet20_sensitivity_n256_s42"
    elif index == 6:
        nodes, n, name = G.heavy_early_resnet20(), 256, "heavyearlyresnet20_sensitivity_n256_s40"
    else:
        raise ValueError("workload index must be 0..10")
    L = G.n_scheme_layers(nodes)
    weights, biases = make_model(nodes, rng)
    n = n if n_images is None else n_images
    images = make_images(n, rng)
    if index == 0:
        schemes = _choice_schemes(rng, 1, L, (32, 8, 4))
    elif index == 1:
        schemes = _choice_schemes(rng, 1, L, (32, 16, 8, 4))
    elif index in (2, 5, 6):
        schemes = np.full((2 * L, L), 32, dtype=np.uint8)
        for i in range(L):
            schemes[2 * i, i] = 8
            schemes[2 * i + 1, i] = 4
    elif index == 3:
        schemes = np.full((16, L), 32, dtype=np.uint8)
        for s in range(16):
            schemes[s, rng.choice(L, 10, replace=False)] = 4
    else:
        schemes = _choice_schemes(rng, 64, L, BITS_ALPHABET)
    if n_schemes is not None:
        schemes = schemes[:n_schemes]
    if seed_index != index:
        name += "_centred"
        if centred:
            biases[-1] = centred_bias(seed_index)
    index = seed_index
    return dict(name=name, index=index, nodes=nodes, desc=G.desc_array(nodes), L=L,
                weights=weights, biases=biases, images=images,
                schemes=np.ascontiguousarray(schemes), chunk=1024)
