"""The C-ABI library loads without a GPU and exports every function include/ep.h
declares; host-side argument validation returns the documented codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ep.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"EP_API\s+[\w\s\*]+?\b(ep_\w+)\s*\(", text)))


@pytest.fixture(scope="module")
def ep():
    from paper_2603_13606_amd import binding, build
    if not build.is_current():
        build.build()
    binding.load()
    return binding


def test_every_declared_function_is_exported(ep):
    names = _declared()
    assert len(names) >= 11 and "ep_dispatch" in names and "ep_layout" in names
    lib = ep.load()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in ep.h but not exported"
    assert sorted(ep.EXPORTS) == names
    for n in names:
        assert callable(getattr(ep, n)), f"binding lacks {n}"


def test_struct_sizes_match_header(ep):
    # config: uint32 + 14 int32; tensor: pointer + 4 int32 + 8 int64
    assert ctypes.sizeof(ep.ep_group_config_t) == 64
    assert ctypes.sizeof(ep.ep_tensor_t) == 8 + 16 + 64
    assert ctypes.sizeof(ep.ep_layout_info_t) == 8 + 7 * 8 + 13 * 8
    assert ctypes.sizeof(ep.ep_group_info_t) == 40 + 7 * 8 + 8 + 6 * 8 + 2 * 8 + 8
    assert ctypes.sizeof(ep.ep_complete_config_t) == 8


def test_error_strings_and_version(ep):
    from paper_2603_13606_amd import build
    assert ep.ep_version() >= 200
    assert ep.ep_build_id() == build.source_id() == build.built_id()
    seen = {ep.error_string(c) for c in range(9)}
    assert len(seen) == 9 and "success" in seen


@pytest.mark.parametrize("kw,code", [
    (dict(num_ranks=3), 1),            # E % R != 0
    (dict(hidden=12), 1),              # 2H not a multiple of 16
    (dict(top_k=0), 1),
    (dict(top_k=65), 1),
    (dict(num_experts=2048), 1),
    (dict(my_rank=2), 1),
    (dict(max_tokens_per_rank=0), 1),
    (dict(mode=5), 1),
    (dict(dtype=1), 4),                # only bf16 tokens
    (dict(staged_buffers=3), 1),
    (dict(dispatch_order=3), 1),
    (dict(dispatch_order=-1), 1),
])
def test_group_create_rejects_bad_config_on_the_host(ep, kw, code):
    args = dict(num_ranks=2, num_experts=8, hidden=256, top_k=2, max_tokens_per_rank=64)
    args.update(kw)
    cfg = ep.make_config(**args)
    with pytest.raises(ep.EpError) as e:
        ep.ep_group_create(cfg, stream=0)
    assert e.value.code == code
    cfg = ep.make_config(2, 8, 256, 2, 64)
    cfg.size = 12
    with pytest.raises(ep.EpError) as e:
        ep.ep_group_create(cfg, stream=0)
    assert e.value.code == ep.EP_ERR_INVALID_ARG


def test_null_arguments(ep):
    lib = ep.load()
    assert lib.ep_group_destroy(None, None) == ep.EP_ERR_INVALID_ARG
    assert lib.ep_handle_destroy(None) == ep.EP_ERR_INVALID_ARG
    assert lib.ep_group_query(None, None) == ep.EP_ERR_INVALID_ARG
    assert lib.ep_dispatch(None, None, 0, None, 0, 0, None) == ep.EP_ERR_INVALID_ARG
    assert lib.ep_combine(None, None, 0, None, 0, 0, None) == ep.EP_ERR_INVALID_ARG
    assert lib.ep_layout(None, None, None, None, None) == ep.EP_ERR_INVALID_ARG
    assert lib.ep_complete(None, None, None) == ep.EP_ERR_INVALID_ARG
    assert lib.ep_group_reset_signals(None, None) == ep.EP_ERR_INVALID_ARG


def test_header_is_plain_c_and_cxx(tmp_path):
    """include/ep.h must compile on its own as C99 and as C++ (no HIP or torch types)."""
    import subprocess
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "use_ep.c"
    src.write_text('#include "ep.h"\nint main(void) { ep_group_config_t c; c.size = sizeof c; '
                   'return ep_version() > 0 && c.size ? 0 : 1; }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)], check=True)
    cxx = tmp_path / "use_ep.cpp"
    cxx.write_text('#include "ep.h"\nint main() { ep_tensor_t t{}; return t.ndim; }\n')
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(cxx)], check=True)


def test_layout_plan_covers_every_entry(ep):
    """Host-side planning: the wave-chunks cover the input, there are at most 512 of them (256
    workgroups of at least two), small inputs fit one workgroup of 16 waves, and up to 512 * 128
    entries a wave keeps its entries in registers (at most two passes)."""
    for n in [0, 1, 63, 64, 65, 1023, 1024, 1025, 4095, 4096, 4097, 16384, 32768, 65536, 65537,
              160000, 262144, 1 << 20, (1 << 28)]:
        passes, chunks = ep.ep_layout_plan(n)
        assert passes >= 1 and 0 <= chunks <= 512
        assert chunks * passes * 64 >= n
        assert (chunks - 1) * passes * 64 < n or n == 0
        if n <= 1024:
            assert passes == 1
        if n <= 4096:
            assert chunks <= 16
        elif n <= 65536:
            assert passes <= 2
    with pytest.raises(ep.EpError):
        ep.ep_layout_plan(-1)


def test_dispatch_plan_covers_the_input_and_fits_the_launch_limits(ep):
    """Host arithmetic of the destination-ordered dispatch: the blocks cover every wave-chunk of
    the layout, the copy launches cover every block, a read pass is planned per launch unless the
    rows were announced to the layout call, and small inputs or the token order plan nothing."""
    import ctypes
    shapes = [(32, 256, 7168, 8, 4096), (64, 256, 7168, 8, 8192), (16, 128, 4096, 8, 4096), (1, 1024, 7168, 16, 4096),
              (8, 8, 64, 1, 9000), (4, 24, 1000, 3, 3000), (64, 1024, 8192, 64, 100000), (2, 2, 8, 2, 5000)]
    for R, E, H, K, T in shapes:
        for order in (ep.EP_ORDER_DESTINATION, ep.EP_ORDER_DESTINATION_RESIDENT):
            cfg = ep.make_config(R, E, H, K, T, dispatch_order=order)
            p = ep.ep_dispatch_plan(cfg, T)
            passes, nwc = ep.ep_layout_plan(T * K)
            if T * K < 8192 or H // 8 < 8:
                assert p.run_order == 0 and p.blocks == 0
                continue
            assert p.run_order == 1
            assert p.group >= 1 and p.blocks * p.group >= nwc > (p.blocks - 1) * p.group
            assert p.block_entries == p.group * passes * 64
            assert 1 <= p.splits and 8 * E * p.splits < 2 ** 31 and p.blocks <= 65535
            slack = 8 if p.slice_units >= 8 else 1  # slices of 8 units or more hold whole 128-byte lines
            assert p.slice_units * 8 >= H // 8 > (p.slice_units - slack) * 8 and (slack == 1 or p.slice_units % 8 == 0)
            assert p.threads_per_piece in (16, 32, 64, 128, 256)
            assert p.launches == -(-p.blocks // p.blocks_per_launch)
            # one slice of a block's tokens stays within 2 MiB (half of an XCD's L2), or the block is
            # a single wave-chunk, which cannot be cut
            assert p.group == 1 or (p.block_entries // K) * (2 * H // 8) <= 2 << 20 or p.block_entries <= 768
            if order == ep.EP_ORDER_DESTINATION:
                assert p.read_passes == p.launches
                tokens_per_launch = -(-p.blocks_per_launch * p.block_entries // K)
                assert p.blocks_per_launch == 1 or tokens_per_launch * 2 * H <= (64 << 20) + 2 * H
                # rows announced to the layout call (at most 64 MiB of them) need no read pass
                first = min(T, (64 << 20) // (2 * H))
                q = ep.ep_dispatch_plan(cfg, T, first)
                assert q.read_passes == p.read_passes - (1 if first >= min(T, tokens_per_launch) else 0)
            else:
                assert p.read_passes == 0 and p.launches == 1
        cfg = ep.make_config(R, E, H, K, T)
        assert ep.ep_dispatch_plan(cfg, T).run_order == 0
    with pytest.raises(ep.EpError):
        ep.ep_dispatch_plan(ep.make_config(2, 8, 256, 2, 64), -1)


def test_combine_plan_follows_rows_and_rounds(ep):
    """Host arithmetic of the combine launch: one 1 KiB segment of a token row per wavefront, two in
    long launches of rows with an even number of segments, the whole row for rows of 14 336 bytes when
    the tokens fill whole rounds (or nearly) of the two-wavefronts-per-SIMD the whole-row kernel holds;
    never for the two-level order; the workgroups cover every (token, piece)."""
    def plan(T, H, cus, **kw):
        return ep.ep_combine_plan(ep.make_config(8, 64, H, 8, max(T, 1), **kw), T, cus)
    slots = 256 * 8
    for T, want in ((4096, 14), (8192, 14), (2048, 14), (2047, 2), (2560, 2), (3072, 2), (3839, 2), (3840, 14), (5120, 2),
                    (6144, 14), (7168, 14), (6500, 14), (100, 1), (1170, 1), (1171, 2), (0, 1)):
        p = plan(T, 7168, 256)
        assert p.segments_per_wavefront == want, (T, p.segments_per_wavefront)
        assert p.whole_row == (want == 14)
        pieces = T * (1 if want == 14 else 14 // want)
        assert p.workgroups == -(-pieces // 4)
        rounds, rest = divmod(T, slots)
        assert (want == 14) == (rounds >= 1 and (rest == 0 or rounds >= 3 or rest * 8 >= slots * 7))
    # other devices: the rounds follow the compute units; an unknown device never takes whole rows
    assert plan(4096, 7168, 304).segments_per_wavefront == 2 and plan(2432 * 2, 7168, 304).segments_per_wavefront == 14
    assert plan(4096, 7168, 0).segments_per_wavefront == 2
    # other rows: 8 segments (two per wavefront when long), 15 segments (odd: one), a ragged 16th segment
    assert plan(4096, 4096, 256).segments_per_wavefront == 2 and plan(100, 4096, 256).segments_per_wavefront == 1
    assert plan(4096, 7680, 256).segments_per_wavefront == 1
    p = plan(4096, 8136, 256)
    assert p.segments_per_wavefront == 2 and p.workgroups == 4096 * 8 // 4
    # the two-level summation order has its own kernel: one segment per wavefront whatever the size
    assert plan(4096, 7168, 256, ranks_per_node=4).segments_per_wavefront == 1
    with pytest.raises(ep.EpError):
        plan(-1, 7168, 256)
    with pytest.raises(ep.EpError):
        ep.ep_combine_plan(ep.make_config(8, 64, 7168, 8, 16), 16, -1)
