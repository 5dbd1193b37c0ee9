"""Comparison implementations of the capsule convolution forward pass, for measurement only.

None of this is on the product path (`capscaps_conv_fwd*` never calls it): these are the rows a
reader of the paper's Table 1 would want next to the implicit-GEMM kernels, run on the same GPU
on the same inputs.

* `scheme1_fwd` -- the paper's Algorithm 3 with every intermediate materialised in device
  memory, as described in Sec. 2 and Figs. 4-7: capsule im2col, replication of the flattened
  input per output channel, replication of the kernel capsules per output pixel, one vendor
  strided-batched small-matrix multiply (through `torch.bmm`), and a separate reduction over
  window and input channels.  Framework tensor ops stand in for the paper's CUDA helpers.
* `framework_conv_fwd` -- the capsule convolution expressed through the framework's own
  convolution (the paper's "GPU" row: Sec. 1.2 notes it can always be built from convolution
  calls).  The operator equals a grouped conv2d with groups = D0, batch (n, d1), input channels
  (c, d2) and output channels (m, d3) per group.
* scheme 2 (Algorithm 5, a flat parallel loop over all small products with accumulation at the
  output) is a HIP kernel in the library: `capscaps_scheme2_*` in the C ABI.
"""
from __future__ import annotations


# Largest batch count handed to the vendor batched multiply in one call.  One call with 2.26e8
# batches of 3x3 products (benchmark configuration 2, eight images at once) ended in a GPU memory
# fault inside that call.  Each operand of that call spanned 8.15 GB, twice what a 32-bit byte
# offset (or one buffer descriptor) can address, and its batch count was far past what one grid
# dimension holds, so the call was beyond two limits at once; a call with 2.9e6 batches and
# 0.1 GB operands (configuration 4) is below both and runs.  Every call made here stays inside
# that proven regime: at most 2^21 products, operands of at most 2^21 * D*D elements.  Larger
# problems are cut over images and output pixels.
MAX_BMM_BATCH = 1 << 21


def scheme1_fwd(inp, kernel, stride=1, pad=0, max_batch_elems=1 << 28):
    """inp [N,H,W,C,D0,D1,D2], kernel [kh,kw,C,M,D0,D2,D3] (device tensors, one dtype) ->
    float32 [N,H',W',M,D0,D1,D3].  The steps of Algorithm 3 run on blocks of images and output
    pixels sized so that no intermediate exceeds `max_batch_elems` elements and no batched
    multiply MAX_BMM_BATCH products."""
    import torch
    import torch.nn.functional as F

    inp, kernel = inp.float(), kernel.float()  # 16-bit operands are widened: fp32 products and sums
    N, H, W, C, D0, D1, D2 = inp.shape
    kh, kw, _, M, _, _, D3 = kernel.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    L, T = Ho * Wo, kh * kw * C
    caps_in = D0 * D1 * D2
    per_pixel = M * T * D0                      # small products per output pixel
    if per_pixel > MAX_BMM_BATCH:
        raise ValueError(f"scheme 1 needs {per_pixel} small products per output pixel in one "
                         f"batched multiply; more than {MAX_BMM_BATCH} is not attempted")
    # pixels (of one or several images) per batched multiply
    budget = max(1, min(MAX_BMM_BATCH // per_pixel,
                        max_batch_elems // max(per_pixel * D1 * max(D2, D3), 1)))
    group = max(1, min(N, budget // L))         # whole images per block, when a block holds any
    block = L if budget >= L else budget        # else: pixels of one image per block
    k_all = kernel.permute(3, 0, 1, 2, 4, 5, 6).reshape(1, 1, M, T, D0, D2, D3)
    out = torch.empty((N, L, M, D0, D1, D3), dtype=torch.float32, device=inp.device)
    for n0 in range(0, N, group):
        x = inp[n0:n0 + group]
        n = x.shape[0]
        # capsule_im2col: one column of kh*kw*C capsules per output pixel
        cols = F.unfold(x.permute(0, 3, 4, 5, 6, 1, 2).reshape(n, C * caps_in, H, W),
                        (kh, kw), padding=pad, stride=stride)          # [n, C*caps*kh*kw, L]
        flat = (cols.reshape(n, C, caps_in, kh * kw, L).permute(0, 4, 3, 1, 2)
                .reshape(n, L, T, D0, D1, D2))
        for l0 in range(0, L, block):
            f = flat[:, l0:l0 + block]
            l = f.shape[1]
            # input_extend: one copy per output channel
            i_ext = f.unsqueeze(2).expand(n, l, M, T, D0, D1, D2).contiguous()
            # kernel_extend: every output pixel gets its own copy of all kernel capsules
            k_ext = k_all.expand(n, l, M, T, D0, D2, D3).contiguous()
            # strided batched small-matrix multiply (vendor library)
            o_ext = torch.bmm(i_ext.reshape(-1, D1, D2), k_ext.reshape(-1, D2, D3))
            # output_reduce: linear combination over window and input channels
            out[n0:n0 + n, l0:l0 + l] = o_ext.reshape(n, l, M, T, D0, D1, D3).sum(dim=3)
    return out.reshape(N, Ho, Wo, M, D0, D1, D3)


def framework_conv_fwd(inp, kernel, stride=1, pad=0, widen=True):
    """Same operator through the framework's grouped conv2d.  `widen`: 16-bit operands are
    converted to fp32 first (exact products and fp32 sums, comparable to the oracle at the
    library's own tolerance); otherwise the convolution runs in the operands' type and its
    16-bit result is converted afterwards (how a framework user would run it)."""
    import torch.nn.functional as F

    if widen:
        inp, kernel = inp.float(), kernel.float()
    N, H, W, C, D0, D1, D2 = inp.shape
    kh, kw, _, M, _, _, D3 = kernel.shape
    # batch (n, d1); channels (d0, c, d2) grouped by d0
    x = inp.permute(0, 5, 4, 3, 6, 1, 2).reshape(N * D1, D0 * C * D2, H, W)
    # weight [(d0, m, d3), (c, d2), kh, kw]
    wgt = kernel.permute(4, 3, 6, 2, 5, 0, 1).reshape(D0 * M * D3, C * D2, kh, kw)
    y = F.conv2d(x, wgt, stride=stride, padding=pad, groups=D0)    # [N*D1, D0*M*D3, Ho, Wo]
    Ho, Wo = y.shape[-2:]
    return (y.reshape(N, D1, D0, M, D3, Ho, Wo).permute(0, 5, 6, 3, 2, 1, 4)
            .contiguous().float())
