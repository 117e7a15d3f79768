"""Helpers shared by the GPU parity tests: move synthetic cases to the device, call the library
through its binding, and bring results back as numpy arrays for comparison with the oracle."""
import numpy as np
import torch

import paper_1801_09449_amd as T


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def words(t: torch.Tensor) -> np.ndarray:
    """Packed device tensor -> uint32 numpy array."""
    return t.cpu().numpy().view(np.uint32)


def run_case(case, want_acc=True, want_packed=True, mfma=False):
    """Run one single-layer case on the GPU (mfma = "i8" or "f4": through tern_conv3d_mfma and
    its filter bank of that kind).  Returns (acc int32 array or None, packed uint32 array or None)."""
    act = T.tern_pack(dev(case.act))
    bank = T.tern_expand_filters(dev(case.wgt), mfma) if mfma else T.tern_pack_filters(dev(case.wgt))
    c_in, c_out = case.act.shape[1], case.wgt.shape[0]
    acc = packed = None
    if want_acc:
        acc = T.tern_conv3d(act, c_in, bank, c_out, case.k, case.stride, case.pad, case.dil, mfma=mfma)
    if want_packed:
        packed = T.tern_conv3d(act, c_in, bank, c_out, case.k, case.stride, case.pad, case.dil,
                               thr_lo=dev(case.lo), thr_hi=dev(case.hi), mfma=mfma)
    torch.cuda.synchronize()
    return (None if acc is None else acc.cpu().numpy(),
            None if packed is None else words(packed))


def bank_layout(w_packed: np.ndarray, c_out: int, c_in: int) -> np.ndarray:
    """Expected filter bank from plane-packed filters [C_out][kd][kh][kw][2][Wd] by pure
    re-indexing.  Plain: [T*nchunk][co_pad][2][wc] with wc = 2 if Wd even else 1.  Tap-packed
    (C_in <= 16, T > 1): [ceil(T/slots)][co_pad][2][1], tap i of a row shifted left by i*shift."""
    wd = (c_in + 31) // 32
    taps = int(np.prod(w_packed.shape[1:4]))
    co_pad = (c_out + 31) // 32 * 32
    if c_in <= 16 and taps > 1:
        shift = 1
        while shift < c_in:
            shift *= 2
        slots = min(32 // shift, taps)
        rows = (taps + slots - 1) // slots
        flat = w_packed.reshape(c_out, taps, 2).astype(np.uint64)       # one word per plane
        bank = np.zeros((rows, co_pad, 2), dtype=np.uint64)
        for t in range(taps):
            bank[t // slots, :c_out] |= flat[:, t] << np.uint64((t % slots) * shift)
        return bank.astype(np.uint32).reshape(-1)
    wc = 2 if wd % 2 == 0 else 1
    nchunk = wd // wc
    flat = w_packed.reshape(c_out, taps, 2, nchunk, wc)            # [co][tap][plane][chunk][q]
    bank = np.zeros((taps, nchunk, co_pad, 2, wc), dtype=np.uint32)
    bank[:, :, :c_out] = np.transpose(flat, (1, 3, 0, 2, 4))
    return bank.reshape(-1)
