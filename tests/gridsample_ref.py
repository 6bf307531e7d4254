"""Second, independent statement of the operator out of a library routine (test helper).

Each tap of Eq. 1 is one call of torch.nn.functional.grid_sample (bilinear, zero
padding, align_corners=True, i.e. integer coordinate = pixel centre) in float64 on
the CPU; the taps are multiplied by the mask and summed.  Autograd of that composition
gives all three gradients.  It shares nothing with oracle/ or with the HIP path.
"""
import torch
import torch.nn.functional as F


def dcnv4_gridsample(x, offset, mask, kernel=3, stride=1, pad=1, dilation=1, offset_scale=1.0):
    """x [N,H,W,C], offset [N,Ho,Wo,G,K,2] (width, height), mask [N,Ho,Wo,G,K] -> y [N,Ho,Wo,C]."""
    N, H, W, C = x.shape
    _, Ho, Wo, G, K, _ = offset.shape
    Cg = C // G
    kh = kw = kernel
    oh = torch.arange(Ho, dtype=x.dtype).view(1, Ho, 1)
    ow = torch.arange(Wo, dtype=x.dtype).view(1, 1, Wo)
    outs = []
    for g in range(G):
        xg = x[..., g * Cg:(g + 1) * Cg].permute(0, 3, 1, 2)          # [N,Cg,H,W]
        acc = 0
        for j in range(kw):            # width index, slow
            for i in range(kh):        # height index, fast
                k = j * kh + i
                hy = oh * stride - pad + i * dilation + offset_scale * offset[:, :, :, g, k, 1]
                wx = ow * stride - pad + j * dilation + offset_scale * offset[:, :, :, g, k, 0]
                # grid_sample wants (x, y) in [-1, 1]; align_corners=True maps -1 -> 0, +1 -> size-1
                gx = 2.0 * wx / (W - 1) - 1.0
                gy = 2.0 * hy / (H - 1) - 1.0
                grid = torch.stack([gx, gy], dim=-1)                   # [N,Ho,Wo,2]
                s = F.grid_sample(xg, grid, mode="bilinear", padding_mode="zeros", align_corners=True)
                acc = acc + s * mask[:, :, :, g, k].unsqueeze(1)
        outs.append(acc.permute(0, 2, 3, 1))
    return torch.cat(outs, dim=-1)


def dcnv4_gridsample_grads(x, offset, mask, grad_y, **kw):
    x = x.clone().requires_grad_(True)
    offset = offset.clone().requires_grad_(True)
    mask = mask.clone().requires_grad_(True)
    y = dcnv4_gridsample(x, offset, mask, **kw)
    (y * grad_y).sum().backward()
    return y.detach(), x.grad, offset.grad, mask.grad
