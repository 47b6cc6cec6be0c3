"""Host-only bounds check of the MLP workers' contraction kernels (csrc/mlp.hip): the index arithmetic
with which every lane of every block addresses the parameter buffers and the work space is restated
here, for every K slice the kernels load (prologue prefetches and in-loop refills included), and the
largest and smallest element offset is asserted to stay inside the array it belongs to -- for every
supported shape class and for the tightest legal buffers (stride = padded d, last worker).  No GPU."""
import itertools

import numpy as np
import pytest

import synth_inputs

K_SLICE = 32


def offsets(n_in, n_hid, n_out):
    W1 = 0
    b1 = n_in * n_hid
    W2 = b1 + n_hid
    b2 = W2 + n_hid * n_out
    return W1, b1, W2, b2


def tile_config(n_hid):
    """(waves along M, waves along N): 64 x 128 block tiles when the hidden width allows, else 64 x 64."""
    return (2, 4) if n_hid % 128 == 0 else (2, 2)


def forward_slices_loaded(n_slices):
    """K slices that the forward product fetches: four in the prologue, two more prefetches clamped to
    the last slice, then iteration s refills with slice s + 6 clamped to the last slice."""
    last = n_slices - 1
    loaded = [0, 1, 2, 3, min(4, last), min(5, last)]
    loaded += [min(s + 6, last) for s in range(n_slices)]
    return sorted(set(loaded))


def backward_slices_loaded(n_slices):
    """Slice 0 in the prologue, slice 1 before the loop, then iteration s loads slice s + 2 for s + 2 < n_slices."""
    return sorted(set([0, 1] + [s + 2 for s in range(n_slices) if s + 2 < n_slices]))


def gemm_operand_ranges(fwd, W, n_in, n_hid, n_out, batch, stride):
    """(min, max+1) element offsets read from X [W][batch][n_in], from the parameter buffer [W][stride]
    (forward: W1) and from dA [W][batch][n_hid] (backward), over all blocks, lanes and loaded slices."""
    nwm, nwn = tile_config(n_hid)
    BM, BN, T = 32 * nwm, 32 * nwn, 64 * nwm * nwn
    PA, PB = (BM * K_SLICE // 4) // T, (K_SLICE * BN // 4) // T
    assert PA * T == BM * K_SLICE // 4 and PB * T == K_SLICE * BN // 4
    a_minor_quads = K_SLICE // 4 if fwd else BM // 4
    a_major_per_pass = T // a_minor_quads
    b_k_per_pass = T // (BN // 4)
    t = np.arange(T, dtype=np.int64)
    a_minor, a_major = (t % a_minor_quads) * 4, t // a_minor_quads
    b_n, b_k = (t % (BN // 4)) * 4, t // (BN // 4)
    M = batch if fwd else n_in
    K = n_in if fwd else batch
    n_slices = K // K_SLICE
    slices = forward_slices_loaded(n_slices) if fwd else backward_slices_loaded(n_slices)
    assert max(slices) == n_slices - 1 and min(slices) == 0
    W1, *_ = offsets(n_in, n_hid, n_out)
    lo = {"X": 2**62, "B": 2**62}
    hi = {"X": -1, "B": -1}
    for worker, m0, n0 in itertools.product((0, W - 1), (0, M - BM), (0, n_hid - BN)):
        xw = worker * batch * n_in
        for s in slices:
            for i in range(PA):
                if fwd:      # a quad is 4 consecutive k of one sample row
                    a = xw + (m0 + a_major) * n_in + a_minor + s * K_SLICE + i * a_major_per_pass * n_in
                else:        # a quad is 4 consecutive input features (rows of X^T) of one sample k
                    a = xw + a_major * n_in + m0 + a_minor + s * K_SLICE * n_in + i * a_major_per_pass * n_in
                lo["X"], hi["X"] = min(lo["X"], a.min()), max(hi["X"], a.max() + 4)
            for i in range(PB):
                base = worker * stride + W1 if fwd else worker * batch * n_hid
                b = base + b_k * n_hid + n0 + b_n + (s * K_SLICE + i * b_k_per_pass) * n_hid
                lo["B"], hi["B"] = min(lo["B"], b.min()), max(hi["B"], b.max() + 4)
    return lo, hi, (BM, BN, T)


SHAPES = [(n_in, n_hid, n_out, batch) for n_in in (128, 256, 3072) for n_hid in (64, 128, 1024)
          for n_out, batch in ((10, 128), (16, 256), (1, 128))]


@pytest.mark.parametrize("n_in,n_hid,n_out,batch", SHAPES)
def test_forward_product_stays_inside_its_operands(n_in, n_hid, n_out, batch):
    W = 3
    d = synth_inputs.mlp_param_count(n_in, n_hid, n_out)
    stride = (d + 3) // 4 * 4                       # the tightest legal row
    lo, hi, _ = gemm_operand_ranges(True, W, n_in, n_hid, n_out, batch, stride)
    assert lo["X"] == 0 and hi["X"] == W * batch * n_in
    # W1 of the last worker ends before b1: nothing is read past the weight matrix, let alone the buffer
    assert lo["B"] == 0 and hi["B"] == (W - 1) * stride + n_in * n_hid <= W * stride


@pytest.mark.parametrize("n_in,n_hid,n_out,batch", SHAPES)
def test_backward_product_and_its_update_stay_inside_their_operands(n_in, n_hid, n_out, batch):
    W = 3
    d = synth_inputs.mlp_param_count(n_in, n_hid, n_out)
    stride = (d + 3) // 4 * 4
    lo, hi, (BM, BN, T) = gemm_operand_ranges(False, W, n_in, n_hid, n_out, batch, stride)
    assert lo["X"] == 0 and hi["X"] == W * batch * n_in
    assert lo["B"] == 0 and hi["B"] == W * batch * n_hid
    # the fused update: tile rows m0 + idx / (BN/4), columns n0 + 4 (idx % (BN/4)) of W1, x / v / stored model
    iters = (BM * BN // 4) // T
    idx = np.arange(iters * T, dtype=np.int64)
    row, col = idx // (BN // 4), (idx % (BN // 4)) * 4
    assert row.max() == BM - 1 and col.max() + 4 == BN
    at_max = (W - 1) * stride + (n_in - BM + row.max()) * n_hid + (n_hid - BN) + col.max() + 4
    assert at_max == (W - 1) * stride + n_in * n_hid <= W * stride
    # the mean is addressed without the worker offset and must fit one row
    assert (n_in - BM + row.max()) * n_hid + (n_hid - BN) + col.max() + 4 <= stride


@pytest.mark.parametrize("n_slices", [4, 8, 12, 96])
def test_slice_schedules_cover_every_slice_and_never_run_past_the_last(n_slices):
    assert forward_slices_loaded(n_slices) == list(range(n_slices))
    assert backward_slices_loaded(n_slices) == list(range(n_slices))


# ---- output-layer kernels --------------------------------------------------------------------------

HEAD_BATCH, HEAD_KEEP, HEAD_SAMPLES = 8, 2, 8          # loads in flight per lane, kept batches, samples (= waves) per block
UPDATE_WAVES, DZ_GROUP, DZ_PITCH = 8, 16, 16           # waves per block, samples per staged group of dZ rows, row pitch of dZ


@pytest.mark.parametrize("n_hid", [64, 192, 1024, 1152, 2944])
@pytest.mark.parametrize("batch", [128, 384, 1024])
def test_output_layer_kernels_stay_inside_their_arrays(n_hid, batch):
    """head: a wave's sample and the hidden units it touches (the kept part of the row first, then batches of
    eight); head_update: a wave's eighth of the batch in groups of 16 samples, one quad of the group's dZ rows
    per lane; the generator groups appended to that launch.  Last worker, tightest buffers."""
    W, n_in = 3, 128
    lanes = np.arange(64, dtype=np.int64)
    # head: blocks of HEAD_SAMPLES waves, one sample each; H is [W][batch][n_hid]
    blocks = (batch + HEAD_SAMPLES - 1) // HEAD_SAMPLES
    samples = np.arange(blocks * HEAD_SAMPLES)
    assert samples[samples < batch].max() == batch - 1                   # waves past the batch take no sample (they load sample 0's row)
    kept = lanes[None, :] + 64 * np.arange(HEAD_BATCH * HEAD_KEEP)[:, None]
    beyond = np.arange(64 * HEAD_BATCH * HEAD_KEEP, max(n_hid, 64 * HEAD_BATCH * HEAD_KEEP) + 64 * HEAD_BATCH)
    touched = np.concatenate([kept.ravel(), beyond])
    touched = touched[touched < n_hid]                                   # every access is guarded by n < n_hid
    assert sorted(set(touched.tolist())) == list(range(n_hid))           # each hidden unit exactly once per sample
    assert (W - 1) * batch * n_hid + (batch - 1) * n_hid + touched.max() < W * batch * n_hid
    # head_update: per wave batch / 8 samples in groups of DZ_GROUP; lane u loads quad u of the group's rows
    per = batch // UPDATE_WAVES
    assert per % DZ_GROUP == 0 and DZ_GROUP * DZ_PITCH == 4 * 64
    first_rows = np.array([s * per + g for s in range(UPDATE_WAVES) for g in range(0, per, DZ_GROUP)])
    dz_elem = ((W - 1) * batch + first_rows[:, None]) * DZ_PITCH + 4 * lanes[None, :] + 3
    assert dz_elem.max() < W * batch * DZ_PITCH and first_rows.max() + DZ_GROUP == batch
    covered = sorted(set((first_rows[:, None] + np.arange(DZ_GROUP)[None, :]).ravel().tolist()))
    assert covered == list(range(batch))                                 # every sample summed exactly once
    # generator groups of 256 threads, UPDATE_WAVES / 4 per block: quads of X [batch][n_in] per worker
    n_quads = batch * n_in // 4
    groups = (n_quads + 255) // 256
    per_block = UPDATE_WAVES // 4
    blocks_per_worker = (groups + per_block - 1) // per_block
    q = (np.arange(blocks_per_worker * per_block)[:, None] * 256 + np.arange(256)[None, :]).ravel()
    q = q[q < n_quads]                                                   # the kernel's own guard
    assert sorted(q.tolist()) == list(range(n_quads))                    # every quad drawn exactly once
