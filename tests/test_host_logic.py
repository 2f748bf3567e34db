"""CPU-only checks of the GPU library's host side: the shared object loads and exports every
symbol include/lp.h declares, argument validation refuses bad calls before any launch, and the
tile geometry the planner hands to the MFMA kernel addresses exactly the pixels the
convolution's definition names (simulated here with the kernel's index formulas).
No GPU compute is called."""
import os
import re

import pytest

import paper_1711_04713_amd as lp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
Q16 = (16, 4, 12)
W16 = (16, 1, 15)
Q8 = (8, 3, 5)
W8 = (8, 1, 7)


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "lp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(lp.lib_path()):
        pytest.skip("liblp.so not built in this checkout (run __graft_entry__.build())")
    lib = lp.load()
    names = _declared_functions()
    assert len(names) >= 15
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(lp.exported_symbols()) == names


def test_status_strings_and_validation_without_gpu():
    assert lp.lp_status_string(0) == "ok"
    d = lp.ConvDesc(1, 8, 8, 16, 16, 3, 3, 1, 1)
    with pytest.raises(lp.LpError) as e:
        lp.lp_conv_packed_bytes(d, (16, 8, 7), W16)          # n != m + f
    assert e.value.status == 1
    with pytest.raises(lp.LpError) as e:
        lp.lp_conv_packed_bytes(lp.ConvDesc(1, 8, 8, 16, 16, 3, 3, 0, 1), Q16, W16)   # stride 0
    assert e.value.status == 1
    with pytest.raises(lp.LpError) as e:
        lp.lp_conv_packed_bytes(lp.ConvDesc(1, 1, 1, 65536, 16, 1, 1, 1, 0), Q16, W16)  # int32 limb sums could overflow
    assert e.value.status == 2
    with pytest.raises(lp.LpError) as e:
        lp.lp_conv_packed_bytes(lp.ConvDesc(4096, 512, 512, 64, 64, 3, 3, 1, 1), Q16, W16)  # >= 2^31 elements
    assert e.value.status == 2
    assert lp.lp_conv_packed_bytes(d, Q16, W16) > 0
    assert lp.lp_fc_packed_bytes(4, 64, 10, Q16, W16) >= 64 * 64 * 2
    assert lp.lp_conv_workspace_bytes(d, Q16, W16) >= 4           # one partial zero count per workgroup
    assert lp.lp_conv_workspace_bytes(lp.ConvDesc(1, 8, 8, 16, 16, 3, 3, 2, 1), Q16, W16) == 0   # direct kernel


def test_path_selection():
    info = lp.lp_conv_plan_info(lp.ConvDesc(2, 16, 16, 64, 64, 3, 3, 1, 1), Q16, W16)
    assert info["path"] == 1 and info["limbs"] == 2 and info["bn"] == 64
    info = lp.lp_conv_plan_info(lp.ConvDesc(2, 16, 16, 64, 128, 3, 3, 1, 1), Q8, W8)
    assert info["path"] == 1 and info["limbs"] == 1 and info["bn"] == 64      # small grid: finer channel tiles
    info = lp.lp_conv_plan_info(lp.ConvDesc(64, 56, 56, 128, 256, 3, 3, 1, 1), Q8, W8)
    assert info["path"] == 1 and info["limbs"] == 1 and info["bn"] == 128
    # 16-bit activations with 8-bit weights ride the two-limb kernel, and so does a 16-bit layer
    # with a tiny window (Cin = 3: the whole 27-long window is one slab); 8-bit activations with
    # 16-bit weights, windows that are neither chunkable nor tiny, and stride 2 take the direct kernel
    assert lp.lp_conv_plan_info(lp.ConvDesc(2, 16, 16, 64, 64, 3, 3, 1, 1), Q16, W8)["path"] == 1
    assert lp.lp_conv_plan_info(lp.ConvDesc(2, 16, 16, 3, 64, 3, 3, 1, 1), Q16, W16)["path"] == 1
    assert lp.lp_conv_plan_info(lp.ConvDesc(2, 16, 16, 64, 64, 3, 3, 1, 1), Q8, W16)["path"] == 0
    assert lp.lp_conv_plan_info(lp.ConvDesc(2, 16, 16, 3, 64, 3, 3, 1, 1), Q8, W8)["path"] == 0
    assert lp.lp_conv_plan_info(lp.ConvDesc(2, 16, 16, 12, 64, 3, 3, 1, 1), Q16, W16)["path"] == 0
    assert lp.lp_conv_plan_info(lp.ConvDesc(2, 16, 16, 64, 64, 3, 3, 2, 1), Q16, W16)["path"] == 0


SHAPES = [
    # N, H, W, Cin, Cout, R, S, pad
    (1, 16, 16, 16, 16, 3, 3, 1),
    (2, 224, 224, 64, 64, 3, 3, 1),
    (3, 112, 112, 64, 128, 3, 3, 1),
    (5, 56, 56, 128, 256, 3, 3, 1),
    (7, 28, 28, 256, 512, 3, 3, 1),
    (32, 14, 14, 512, 512, 3, 3, 1),
    (3, 13, 11, 32, 48, 3, 3, 1),
    (2, 9, 20, 16, 200, 5, 5, 2),
    (2, 18, 18, 64, 64, 7, 7, 3),
    (4, 10, 10, 64, 64, 3, 3, 0),
    (2, 12, 12, 64, 64, 1, 1, 0),
    (2, 6, 40, 32, 32, 3, 5, 2),
    (300, 1, 1, 4096, 1000, 1, 1, 0),      # FC as a 1x1 conv over a 1x1 image
    (130, 2, 2, 64, 64, 3, 3, 1),          # many image boundaries inside one tile
    (1, 3, 200, 16, 16, 3, 3, 1),
    (2, 224, 224, 3, 64, 3, 3, 1),         # first VGG16 layer: flat-window variant
    (3, 20, 20, 1, 16, 7, 7, 3),
]


@pytest.mark.parametrize("N,H,W,Cin,Cout,R,S,pad", SHAPES)
def test_tile_geometry_addresses_the_right_pixels(N, H, W, Cin, Cout, R, S, pad):
    """Re-run the kernel's table construction for every tile: each output pixel is produced by
    exactly one tile row, and tap (r, s) of that row reads input pixel (y+r-pad, x+s-pad) of the
    same image, or the zero code outside the image; every staged index stays inside the patch."""
    info = lp.lp_conv_plan_info(lp.ConvDesc(N, H, W, Cin, Cout, R, S, 1, pad), Q16, W16)
    assert info["path"] == 1
    RH, TW, PRA, PW = info["tile_rows"], info["tile_cols"], info["patch_rows"], info["patch_cols"]
    Ho, Wo, Hp = H + 2 * pad - R + 1, W + 2 * pad - S + 1, H + 2 * pad
    FR = N * Ho
    assert RH * TW <= 128 and PW == TW + S - 1
    tiles_r, tiles_c = -(-FR // RH), -(-Wo // TW)
    assert info["tiles_m"] == tiles_r * tiles_c
    assert info["lds_bytes"] <= 80 * 1024
    NPIXA = PRA * PW
    pitch, pix = info["patch_pitch"], info["patch_pixel"]
    if info["kernel"] == lp.LP_KERNEL_ROWS:
        # dense pixels of Cin bytes per limb; 16 lanes = 16 consecutive tile rows read the same
        # 16-byte slot of their window's first pixel (every piece of every window row shifts them
        # all by the same amount)
        assert Cin in (16, 32, 48) and pix == Cin and pitch % 16 == 0 and PW * pix <= pitch < PW * pix + 256
        assert info["lds_bytes"] <= 40 * 1024
        worst = 0
        for m0 in range(0, RH * TW, 16):
            groups = {}
            for m in range(m0, min(m0 + 16, RH * TW)):
                g = (((m // TW) * pitch + (m % TW) * pix) // 16) % 16
                groups[g] = groups.get(g, 0) + 1
            worst = max(worst, max(groups.values()))
        assert worst <= (1 if Cin == 16 and TW in (1, 2, 4, 8, 16) else 3)
    elif Cin >= 16:
        assert pix == 80 and pitch % 16 == 0 and PW * pix <= pitch < PW * pix + 256
        # fragment reads: 16 lanes = 16 consecutive tile rows m read the same 16-byte slot q of
        # their pixel (patch_row, patch_col) at tap (r, s), stored at patch_row * pitch +
        # patch_col * 80 + 16 * q.  The 64 LDS banks serve 256 bytes per pass: count lanes that
        # share a 16-byte bank group.  Power-of-two tile widths must be conflict-free; odd widths
        # may keep a 2-way conflict.
        worst = 0
        for r in range(R):
            for s_ in range(S):
                for m0 in range(0, RH * TW, 16):
                    groups = {}
                    for m in range(m0, min(m0 + 16, RH * TW)):
                        prow, pcol = m // TW + r, m % TW + s_
                        g = ((prow * pitch + pcol * pix) // 16) % 16
                        groups[g] = groups.get(g, 0) + 1
                    worst = max(worst, max(groups.values()))
        assert worst <= (1 if TW in (1, 2, 4, 8, 16, 32, 64, 128) else 2)
    seen = set()
    # every tile when there are few; otherwise the first, the last and a spread in between
    rows = range(tiles_r) if tiles_r <= 64 else sorted(set([0, 1, tiles_r - 2, tiles_r - 1] + list(range(0, tiles_r, max(1, tiles_r // 50)))))
    for tile_r in rows:
        fr0 = tile_r * RH
        vr0 = (fr0 // Ho) * Hp + fr0 % Ho
        for tile_c in range(tiles_c):
            x0 = tile_c * TW
            tab = []
            for p in range(NPIXA):
                pr, pc = divmod(p, PW)
                vr = vr0 + pr
                n, iy, ix = vr // Hp, vr % Hp - pad, x0 - pad + pc
                ok = n < N and 0 <= iy < H and 0 <= ix < W
                tab.append((n * H + iy) * W + ix if ok else -1)
            for m in range(128):
                j, t = divmod(m, TW)
                fr, xo = fr0 + j, x0 + t
                if not (j < RH and fr < FR and xo < Wo):
                    continue
                n, yo = divmod(fr, Ho)
                out = fr * Wo + xo
                assert out not in seen
                seen.add(out)
                base = ((fr // Ho) * Hp + fr % Ho - vr0) * PW + t
                assert 0 <= base and base + (R - 1) * PW + (S - 1) < NPIXA
                for r in (0, R // 2, R - 1):
                    for s in (0, S // 2, S - 1):
                        iy, ix = yo + r - pad, xo + s - pad
                        want = (n * H + iy) * W + ix if (0 <= iy < H and 0 <= ix < W) else -1
                        assert tab[base + r * PW + s] == want
    if tiles_r <= 64:
        assert len(seen) == FR * Wo


@pytest.mark.parametrize("N,H,W,Cin,Cout,R,S,pad", SHAPES + [(32, 56, 56, 256, 256, 3, 3, 1), (32, 28, 28, 512, 512, 3, 3, 1)])
def test_launch_geometry_covers_every_tile_and_slab_once(N, H, W, Cin, Cout, R, S, pad):
    """Re-run the kernel's decoding of a workgroup id into (tile, part): every tile is computed
    either by one whole workgroup or by `split` parts whose slab ranges partition the reduction."""
    info = lp.lp_conv_plan_info(lp.ConvDesc(N, H, W, Cin, Cout, R, S, 1, pad), Q16, W16)
    total = info["tiles_m"] * info["tiles_n"]
    split, grid = info["split"], info["workgroups"]
    flat = info["kernel"] != lp.LP_KERNEL_PATCH        # one slab: the flat-window and window-row kernels
    nslabs = 1 if flat else -(-Cin // 64) * R * S
    per_xcd = -(-total // 8)
    assert grid % 8 == 0 and 1 <= split <= max(1, min(nslabs, 8))
    if split == 1:
        full = per_xcd
        assert grid == 8 * per_xcd
    else:
        assert (per_xcd * split - grid // 8) % (split - 1) == 0
        full = (per_xcd * split - grid // 8) // (split - 1)
        assert 0 <= full < per_xcd
    covered = {}
    for b in range(grid):
        xcd, slot = b & 7, b >> 3
        tl, part, nparts = slot, 0, 1
        if slot >= full:
            u = slot - full
            tl, part, nparts = full + u // split, u % split, split
        wi = xcd * per_xcd + tl
        if tl >= per_xcd or wi >= total:
            continue
        s0, s1 = part * nslabs // nparts, (part + 1) * nslabs // nparts
        assert s0 < s1
        covered.setdefault(wi, []).append((s0, s1))
    assert sorted(covered) == list(range(total))
    for wi, ranges in covered.items():
        ranges.sort()
        assert ranges[0][0] == 0 and ranges[-1][1] == nslabs
        assert all(a[1] == b[0] for a, b in zip(ranges, ranges[1:]))
    ws = lp.lp_conv_workspace_bytes(lp.ConvDesc(N, H, W, Cin, Cout, R, S, 1, pad), Q16, W16)
    tails = 8 * (per_xcd - full)
    assert ws >= grid * 4 + (tails * split * (128 * info["bn"] * 3 * 4 + 512) if split > 1 else 0)


def test_pool_check_lists_every_condition_of_the_fused_pool():
    """lp_conv_pool_check answers on the host what lp_conv_fwd would say to d.pool = 1."""
    d = lp.ConvDesc(32, 224, 224, 64, 64, 3, 3, 1, 1, 1)
    assert lp.lp_conv_pool_check(d, Q16, W16, (16, 6, 10))
    assert not lp.lp_conv_pool_check(d, Q16, W16, (16, 6, 10), relu=False)
    assert not lp.lp_conv_pool_check(d, Q16, W16, (16, 6, 10), r=lp.LP_ROUND_NEAREST_EVEN)
    assert not lp.lp_conv_pool_check(d, Q16, W16, (8, 6, 2))                       # 8-bit codes out
    assert not lp.lp_conv_pool_check(d, Q16, W16, (16, 6, 10), qb=(16, 15, 1))     # bias shift beyond 24 bits
    assert lp.lp_conv_pool_check(d, Q16, W16, (16, 6, 10), qb=(16, 4, 12))
    wide = lp.ConvDesc(2, 16, 16, 1024, 64, 3, 3, 1, 1, 1)                         # K = 9216 > 8192
    try:
        assert not lp.lp_conv_pool_check(wide, Q16, W16, (16, 6, 10))
    except lp.LpError as e:                                                        # or no poolable tiling at all
        assert e.status == 2
