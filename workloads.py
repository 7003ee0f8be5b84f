"""Seeded synthetic inputs for the workload configurations.

Input generation only: no arithmetic of the method lives here (no split, no
gather, no loss, no update).  Both the test/bench side that drives the HIP
library and the side that drives the CPU oracle draw their inputs from this
module so that they see identical arrays.

Every generator takes `scale` arguments so that tests can run the same recipe
at sizes the CPU oracle finishes in seconds; the defaults are the full sizes.
Seeds follow rng = numpy.random.default_rng(171004162 + config_number).
"""
import numpy as np

SEED_BASE = 171004162


def rng_for(cfg, salt=0):
    return np.random.default_rng(SEED_BASE + cfg + 1000 * salt)


def mlp_param_count(dims):
    return sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))


def mlp_init(dims, rng):
    """He-normal weights W_l ~ N(0, 2/fan_in), zero biases, as one flat float32
    array in the order W_1, b_1, W_2, b_2, ... with W_l [fan_in x fan_out]
    row-major."""
    parts = []
    for l in range(len(dims) - 1):
        k, n = dims[l], dims[l + 1]
        parts.append((rng.standard_normal((k, n)) * np.sqrt(2.0 / k)).astype(np.float32).ravel())
        parts.append(np.zeros(n, dtype=np.float32))
    return np.concatenate(parts)


def config1(n_data=4096, batch=256):
    """Tiny MLP step: data ~N(0,1) fp32 [n_data x 784], labels U{0..9}, MLP
    784-256-10, batch = prefix of a seeded permutation, 2 workers x 4 slices,
    momentum SGD lr 0.01 m 0.9, fp32."""
    rng = rng_for(1)
    dims = [784, 256, 10]
    return dict(
        name="cfg1_tiny_mlp", dims=dims, compute="f32",
        data=rng.standard_normal((n_data, 784)).astype(np.float32),
        labels=rng.integers(0, 10, n_data).astype(np.int32),
        idx=rng.permutation(n_data)[:batch].astype(np.int32),
        theta=mlp_init(dims, rng), n_workers=2, n_slices=4,
        lr=0.01, momentum=0.9, weight_decay=0.0)


def config2(n_data=50000, batch=1024, dims=(3072, 1024, 1024, 10), n_workers=8, n_slices=4,
            n_index_sets=1):
    """Wide MLP step: data U[0,1) fp32 [n_data x 3072], labels U{0..9}, MLP
    3072-1024-1024-10, batch of seeded random indices (duplicates possible),
    8 worker shares x 4 slices, bf16 GEMM inputs / fp32 accumulate."""
    rng = rng_for(2)
    dims = list(dims)
    data = rng.random((n_data, dims[0]), dtype=np.float32)
    labels = rng.integers(0, dims[-1], n_data).astype(np.int32)
    idx_sets = [rng.integers(0, n_data, batch).astype(np.int32) for _ in range(n_index_sets)]
    return dict(
        name="cfg2_wide_mlp", dims=dims, compute="bf16", data=data, labels=labels,
        idx=idx_sets[0], idx_sets=idx_sets, theta=mlp_init(dims, rng),
        n_workers=n_workers, n_slices=n_slices, lr=0.01, momentum=0.9, weight_decay=0.0)


def resnet50_tensor_shapes():
    """Shapes of the 161 parameter tensors of ResNet-50, from the architecture
    rule: 7x7 stem of 64 filters; bottleneck stages of [3,4,6,3] blocks with
    widths 64/128/256/512 and expansion 4, a 1x1 projection in the first block
    of each stage; a scale and a shift vector after every convolution; a
    2048x1000 classifier with bias."""
    shapes = []

    def conv(cout, cin, k):
        shapes.append((cout, cin, k, k))
        shapes.append((cout,))
        shapes.append((cout,))

    conv(64, 3, 7)
    cin = 64
    for blocks, width in zip((3, 4, 6, 3), (64, 128, 256, 512)):
        for b in range(blocks):
            conv(width, cin, 1)
            conv(width, width, 3)
            conv(4 * width, width, 1)
            if b == 0:
                conv(4 * width, cin, 1)
            cin = 4 * width
    shapes.append((2048, 1000))
    shapes.append((1000,))
    return shapes


def config3(n_params=None, n_workers=8):
    """ResNet-50-sized gradient reduction: n_workers flat fp32 buffers ~N(0,
    sigma=1e-3) laid out as the 161 tensors above; p ~N(0, 0.05), v = 0; one
    scalar loss per worker; lr 0.1, m 0.9, wd 1e-4."""
    rng = rng_for(3)
    shapes = resnet50_tensor_shapes()
    sizes = [int(np.prod(s)) for s in shapes]
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P = int(offsets[-1]) if n_params is None else int(n_params)
    grads = [(rng.standard_normal(P, dtype=np.float32) * np.float32(1e-3)) for _ in range(n_workers)]
    return dict(
        name="cfg3_resnet50_reduce", shapes=shapes, offsets=offsets, n_params=P,
        grads=grads, p=(rng.standard_normal(P, dtype=np.float32) * np.float32(0.05)),
        v=np.zeros(P, dtype=np.float32),
        losses=rng.random(n_workers, dtype=np.float32) * np.float32(7.0),
        n_workers=n_workers, lr=0.1, momentum=0.9, weight_decay=1e-4)


def config4(n_data=50000, batch=256, chw=(3, 224, 224), n_workers=8, n_index_sets=1):
    """Input-indexing gather: uint8 images U{0..255}, labels U{0..999}, batch
    of seeded random indices, per-channel mean/std on the 0..255 scale."""
    rng = rng_for(4)
    c, h, w = chw
    data = rng.integers(0, 256, (n_data, c, h, w), dtype=np.uint8)
    labels = rng.integers(0, 1000, n_data).astype(np.int32)
    idx_sets = [rng.integers(0, n_data, batch).astype(np.int32) for _ in range(n_index_sets)]
    mean = (np.array([0.485, 0.456, 0.406, 0.45][:c] + [0.45] * max(0, c - 4)) * 255.0).astype(np.float32)
    std = (np.array([0.229, 0.224, 0.225, 0.225][:c] + [0.225] * max(0, c - 4)) * 255.0).astype(np.float32)
    return dict(name="cfg4_gather", data=data, labels=labels, idx=idx_sets[0], idx_sets=idx_sets,
                mean=mean, std=std, n_workers=n_workers)


def config5(rows=65536, classes=1000, n_slices=64, salt=0):
    """Slice-aggregation stress: logits ~N(0, sigma=2) fp32 [rows x classes],
    labels uniform, n_slices slices."""
    rng = rng_for(5, salt)
    logits = rng.standard_normal((rows, classes), dtype=np.float32) * np.float32(2.0)
    labels = rng.integers(0, classes, rows).astype(np.int32)
    return dict(name="cfg5_slice_aggregation", logits=logits, labels=labels, n_slices=n_slices)


def convblock_param_count(shape):
    H, W, cin, cout, classes = shape
    return 9 * cin * cout + 2 * cout + cout * classes + classes


def convblock_init(shape, rng):
    """One flat float32 array: Wc [3 x 3 x C_in x C_out] ~ N(0, 2/(9 C_in)),
    gamma ~ U[0.5, 1.5), beta ~ N(0, 0.1^2), Wf [C_out x classes] ~
    N(0, 1/C_out), bf = 0."""
    H, W, cin, cout, classes = shape
    return np.concatenate([
        (rng.standard_normal(9 * cin * cout) * np.sqrt(2.0 / (9 * cin))).astype(np.float32),
        (0.5 + rng.random(cout)).astype(np.float32),
        (rng.standard_normal(cout) * 0.1).astype(np.float32),
        (rng.standard_normal(cout * classes) * np.sqrt(1.0 / cout)).astype(np.float32),
        np.zeros(classes, dtype=np.float32)])


def config6(n_data=256, batch=64, shape=(56, 56, 64, 64, 1000), n_workers=8, n_slices=1, compute="bf16"):
    """Convolution + batch-normalisation block at the shape of the 3x3
    convolutions in the first stage of ResNet-50 (56 x 56 positions, 64 -> 64
    channels; the scaling study's batch of 64 images over 8 workers, no input
    slicing): images ~N(0,1) fp32 stored channels-last as rows of H*W*C_in
    values (the study's inputs are random single-precision arrays), labels
    U{0..classes-1}, batch of seeded random indices."""
    rng = rng_for(6)
    H, W, cin, cout, classes = shape
    data = rng.standard_normal((n_data, H * W * cin), dtype=np.float32)
    labels = rng.integers(0, classes, n_data).astype(np.int32)
    idx = rng.integers(0, n_data, batch).astype(np.int32)
    return dict(name="cfg6_conv_bn_block", shape=tuple(shape), compute=compute, data=data, labels=labels,
                idx=idx, theta=convblock_init(shape, rng), n_workers=n_workers, n_slices=n_slices,
                eps=1e-5, lr=0.1, momentum=0.9, weight_decay=1e-4)
