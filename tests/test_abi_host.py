"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares, and turns bad
arguments into error codes before any HIP call."""
import ctypes as C
import os
import re

import pytest

from paper_2509_02480_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000  # never dereferenced: validation fails first, or n == 0
FAKE_PAGE = 0x7F1000000000


def header_functions():
    text = open(os.path.join(ROOT, "include", "mlpo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mlpo_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = header_functions()
    assert set(names) == set(B.EXPORTS)
    dll = C.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(dll, n) is not None


def test_version_and_workspace_size():
    assert B.mlpo_version() >= 100
    assert B.mlpo_norm_workspace_bytes() >= 4096


def sg(n=8, tier=0, **kw):
    d = dict(p=FAKE, m=FAKE + 4096, v=FAKE + 8192, g=FAKE + 12288, p16=FAKE + 16384)
    d.update(kw)
    return B.SubgroupC(d["p"], d["m"], d["v"], d["g"], d["p16"], n, tier, d.get("tile_elems", 0),
                       d.get("half_format", 0), d.get("lead", 0))


def expect(code, fn, *a, **k):
    with pytest.raises(B.MlpoError) as e:
        fn(*a, **k)
    assert e.value.code == code, str(e.value)
    assert str(e.value)


@pytest.mark.parametrize("kw", [dict(lr=-1.0), dict(lr=float("nan")), dict(beta1=1.0), dict(beta2=-0.1),
                                dict(eps=float("inf")), dict(weight_decay=-1e-3)])
def test_bad_hyperparameters(kw):
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [], B.HParams(**kw), 1)


def test_bad_step_and_pointers():
    hp = B.HParams()
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [], hp, 0)
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(p=0)], hp, 1)
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(g=0)], hp, 1)
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(p=FAKE + 2)], hp, 1)      # fp32 not 4-byte aligned
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(g=FAKE + 1)], hp, 1)      # bf16 not 2-byte aligned
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(tier=1)], hp, 1)          # host tier needs the pipeline
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(tier=7)], hp, 1)
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg()], hp, 1, scalars=FAKE + 4)  # scalars not 16-byte aligned
    # tiled state: T a multiple of 1024, 256-byte aligned buffer, m and v where the layout puts them
    T = 2048
    ok = B.tiled_subgroup(FAKE, FAKE + (1 << 20), FAKE + (2 << 20), n=0, tile_elems=T)
    B.mlpo_adamw_step([ok], hp, 1)                                        # n == 0: nothing dereferenced
    for bad in (B.tiled_subgroup(FAKE, FAKE + (1 << 20), FAKE + (2 << 20), n=8, tile_elems=1000),
                B.tiled_subgroup(FAKE + 64, FAKE + (1 << 20), FAKE + (2 << 20), n=8, tile_elems=T),
                B.tiled_subgroup(FAKE, FAKE + (1 << 20) + 2, FAKE + (2 << 20), n=8, tile_elems=T),
                B.SubgroupC(FAKE, FAKE + 4 * T, FAKE + 8 * T + 4, FAKE + (1 << 20), FAKE + (2 << 20), 8, 0, T),
                B.SubgroupC(FAKE, FAKE + 4 * T, FAKE + 8 * T, FAKE + (1 << 20), FAKE + (2 << 20), 8, 0, -1024)):
        expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [bad], hp, 1)
    # nothing to do is not an error
    B.mlpo_adamw_step([], hp, 1)
    rc = B.lib().mlpo_adamw_step(None, -1, C.byref(hp.c()), 1, None, None)
    assert rc == B.MLPO_EINVAL
    rc = B.lib().mlpo_adamw_step(None, 1, C.byref(hp.c()), 1, None, None)
    assert rc == B.MLPO_EINVAL
    rc = B.lib().mlpo_adamw_step(None, 0, None, 1, None, None)
    assert rc == B.MLPO_EINVAL


def test_norm_argument_errors():
    ws = B.mlpo_norm_workspace_bytes()
    expect(B.MLPO_EINVAL, B.mlpo_grad_unscale_norm, [sg()], 0.0, 0.0, FAKE, ws, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_grad_unscale_norm, [sg()], float("inf"), 0.0, FAKE, ws, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_grad_unscale_norm, [sg()], 1.0, float("nan"), FAKE, ws, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_grad_unscale_norm, [sg()], 1.0, 0.0, 0, ws, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_grad_unscale_norm, [sg()], 1.0, 0.0, FAKE + 64, ws, FAKE)
    expect(B.MLPO_ENOMEM, B.mlpo_grad_unscale_norm, [sg()], 1.0, 0.0, FAKE, ws - 1, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_grad_unscale_norm, [sg()], 1.0, 0.0, FAKE, ws, 0)
    expect(B.MLPO_EINVAL, B.mlpo_grad_unscale_norm, [sg()], 1.0, 0.0, FAKE, ws, FAKE + 8)
    expect(B.MLPO_EINVAL, B.mlpo_grad_unscale_norm, [sg(g=0)], 1.0, 0.0, FAKE, ws, FAKE)


def cfg(n_slots=3, staging=FAKE, staging_bytes=1 << 30, chunk=0):
    return B.stream_cfg(n_slots, staging, staging_bytes, None, None, None, chunk)


def test_stream_argument_errors():
    hp = B.HParams()
    host = [sg(n=1000, tier=1), sg(n=500, tier=0)]
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, cfg(n_slots=0))
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, cfg(n_slots=B.MAX_SLOTS + 1))
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, cfg(chunk=6))
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, cfg(staging=0))
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, cfg(staging=FAKE + 16))
    expect(B.MLPO_ENOMEM, B.mlpo_stream_update, host, None, hp, 1, None, cfg(staging_bytes=3 * 12 * 1000 - 1))
    tiled = [B.tiled_subgroup(FAKE, FAKE + (1 << 30), FAKE + (2 << 30), n=5000, tier=1, tile_elems=2048)]
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, tiled, None, hp, 1, None, cfg(chunk=1024))   # not a multiple of T
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, [0, 0], hp, 1, None, cfg())
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, [0, 2], hp, 1, None, cfg())
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 0, None, cfg())
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, B.HParams(beta1=2.0), 1, None, cfg())
    bad_mode = cfg()
    bad_mode.mode = 2
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, bad_mode)
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, B.direct_cfg(None, None, 5000))
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, B.direct_cfg(None, None, -1))
    res = cfg()
    res.reserved = 1
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, res)
    # slot cache: staged mode, a struct that is zero or ours, slots sized for whole subgroups
    cache = B.SlotCacheC()
    small = B.mlpo_stream_staging_bytes(host, 3, 512)
    assert small < B.mlpo_stream_staging_bytes(host, 3, B.CHUNK_WHOLE)
    with_cache = B.stream_cfg(3, FAKE, small, None, None, None, 512, cache=cache)
    expect(B.MLPO_ENOMEM, B.mlpo_stream_update, host, None, hp, 1, None, with_cache)   # slots hold whole subgroups
    d = B.direct_cfg(None, None, 8)
    d.cache = C.pointer(cache)
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None, d)                     # direct mode
    junk = B.SlotCacheC()
    junk.magic = 12345
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, host, None, hp, 1, None,
           B.stream_cfg(3, FAKE, 1 << 30, None, None, None, 0, cache=junk))
    expect(B.MLPO_EINVAL, B.mlpo_stream_flush, host, cfg())                                     # no cache
    B.mlpo_stream_flush(host, B.stream_cfg(3, FAKE, 1 << 30, None, None, None, 0, cache=B.SlotCacheC()))  # unused: ok
    rc = B.lib().mlpo_stream_update(None, 0, None, C.byref(hp.c()), 1, None, None, None)
    assert rc == B.MLPO_EINVAL
    # an empty list is a no-op that counts as applied
    assert B.mlpo_stream_update([], None, hp, 1, None, cfg()) is True


def test_staging_size_formula():
    host = [sg(n=1000, tier=1), sg(n=4001, tier=1), sg(n=10 ** 6, tier=0)]
    assert B.mlpo_stream_staging_bytes(host, 3) == 3 * 12 * 4032          # arrays rounded to 64 elements (256 bytes)
    assert B.mlpo_stream_staging_bytes(host, 2, 1024) == 2 * 12 * 1024
    assert B.mlpo_stream_staging_bytes(host, 2, 8000) == 2 * 12 * 4032
    assert B.mlpo_stream_staging_bytes([sg(tier=0)], 4) == 0
    tiled = [B.tiled_subgroup(FAKE, FAKE + (1 << 30), FAKE + (2 << 30), n=5000, tier=1, tile_elems=2048)]
    assert B.mlpo_stream_staging_bytes(tiled, 2) == 2 * 12 * 6144         # whole layout tiles
    assert B.mlpo_stream_staging_bytes(tiled, 2, 4096) == 2 * 12 * 4096
    assert B.mlpo_state_floats(5000, 2048) == 3 * 6144 and B.mlpo_state_floats(5000, 0) == 15000
    assert B.mlpo_state_floats(0, 2048) == 0 and B.mlpo_state_floats(2048, 2048) == 3 * 2048


def test_pack_argument_errors():
    expect(B.MLPO_EINVAL, B.mlpo_state_pack, FAKE, FAKE, FAKE, 10, 1000, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_state_pack, FAKE, FAKE, FAKE, 10, 0, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_state_pack, FAKE, 0, FAKE, 10, 1024, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_state_unpack, FAKE + 2, 10, 1024, FAKE, FAKE, FAKE)
    B.mlpo_state_pack(0, 0, 0, 0, 1024, 0)          # nothing to do


def test_timing_switch_and_shutdown():
    B.mlpo_kernel_timing(True)
    assert B.mlpo_kernel_times(0) == []         # nothing launched, nothing recorded
    expect(B.MLPO_EINVAL, B.mlpo_kernel_times, 5)
    expect(B.MLPO_EINVAL, B.mlpo_kernel_times, -1)
    B.mlpo_kernel_timing(False)
    B.mlpo_shutdown()


def test_grad_accumulate_argument_errors():
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate, 0, FAKE, 16)
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate, FAKE, 0, 16)
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate, FAKE + 1, FAKE + 4096, 16)          # not 2-byte aligned
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate, FAKE, FAKE + 30, 16)                # ranges overlap
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate, FAKE + 30, FAKE, 16)
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate, FAKE, FAKE + 4096, 16, blocks=-1)
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate, FAKE, FAKE + 4096, 16, blocks=5000)
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate, FAKE, FAKE + (1 << 50), (1 << 44) + 1)
    B.mlpo_grad_accumulate(0, 0, 0)                                                   # n = 0: nothing to do


def test_staging_size_counts_host_side_gradients():
    # planar: 3 arrays of round_up(n, 64) floats; with the gradients on the host the slot also holds round_up(n, 128)
    # bf16 values behind them
    state_only = [sg(n=1000, tier=B.TIER_HOST)]
    with_grads = [sg(n=1000, tier=B.TIER_HOST_GRADS)]
    assert B.mlpo_stream_staging_bytes(state_only, 2, 0) == 2 * 3 * 1024 * 4
    assert B.mlpo_stream_staging_bytes(with_grads, 2, 0) == 2 * (3 * 1024 * 4 + 1024 * 2)
    assert B.mlpo_stream_staging_bytes(with_grads, 3, 400) == 3 * (3 * 448 * 4 + 512 * 2)
    tiled = [B.tiled_subgroup(FAKE, FAKE + (1 << 30), FAKE + (2 << 30), n=5000, tier=B.TIER_HOST_GRADS, tile_elems=2048)]
    assert B.mlpo_stream_staging_bytes(tiled, 1, 0) == 3 * 6144 * 4 + 5120 * 2
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(tier=B.TIER_HOST_GRADS)], B.HParams(), 1)


def test_accumulate_norm_argument_errors():
    ws = B.mlpo_norm_workspace_bytes()
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate_norm, FAKE, FAKE + 4096, 16, False, 0, 1.0, 0, ws, True)
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate_norm, FAKE, FAKE + 4096, 16, False, 0, 1.0, FAKE + 64, ws, True)
    expect(B.MLPO_ENOMEM, B.mlpo_grad_accumulate_norm, FAKE, FAKE + 4096, 16, False, 0, 1.0, FAKE, ws - 1, True)
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate_norm, FAKE, FAKE + 4096, 16, False, 0, 0.0, FAKE, ws, True)
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate_norm, FAKE, FAKE + 8, 16, False, 0, 1.0, FAKE, ws, True)   # overlap
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate_norm, 0, FAKE + 4096, 16, False, 0, 1.0, FAKE, ws, True)
    B.mlpo_grad_accumulate_norm(0, 0, 0, False, 0, 1.0, FAKE, ws, False)          # nothing to add, nothing to reset
    expect(B.MLPO_EINVAL, B.mlpo_grad_norm_finish, 0, ws, 1.0, 0.0, FAKE)
    expect(B.MLPO_ENOMEM, B.mlpo_grad_norm_finish, FAKE, 16, 1.0, 0.0, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_grad_norm_finish, FAKE, ws, float("nan"), 0.0, FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_grad_norm_finish, FAKE, ws, 1.0, float("nan"), FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_grad_norm_finish, FAKE, ws, 1.0, 0.0, 0)
    expect(B.MLPO_EINVAL, B.mlpo_grad_norm_finish, FAKE, ws, 1.0, 0.0, FAKE + 8)


def test_binding_structs_match_the_header(tmp_path):
    """sizeof and the offsets of the last fields, printed by a C program that includes mlpo.h, against the ctypes
    mirrors in the binding."""
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text('''
#include <stdio.h>
#include <stddef.h>
#include "mlpo.h"
int main(void) {
    printf("%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\\n", sizeof(mlpo_adamw_hparams), sizeof(mlpo_subgroup),
           sizeof(mlpo_step_scalars), sizeof(mlpo_slot_cache), sizeof(mlpo_stream_cfg), sizeof(mlpo_file_extent),
           sizeof(mlpo_file_stats), offsetof(mlpo_stream_cfg, flush_to), offsetof(mlpo_slot_cache, hits),
           offsetof(mlpo_subgroup, tile_elems));
    printf("%zu %zu %zu %zu %zu %zu\\n", sizeof(mlpo_flush_target), offsetof(mlpo_flush_target, file),
           sizeof(mlpo_path_stats), offsetof(mlpo_path_stats, stats), offsetof(mlpo_stream_cfg, path_stats),
           offsetof(mlpo_stream_cfg, path_stats_cap));
    return 0;
}
''')
    exe = tmp_path / "sizes"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.check_call(["gcc", "-I", inc, "-o", str(exe), str(src)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    want = [C.sizeof(B.HParamsC), C.sizeof(B.SubgroupC), C.sizeof(B.StepScalarsC), C.sizeof(B.SlotCacheC),
            C.sizeof(B.StreamCfgC), C.sizeof(B.FileExtentC), C.sizeof(B.FileStatsC), B.StreamCfgC.flush_to.offset,
            B.SlotCacheC.hits.offset, B.SubgroupC.tile_elems.offset, C.sizeof(B.FlushTargetC),
            B.FlushTargetC.file.offset, C.sizeof(B.PathStatsC), B.PathStatsC.stats.offset,
            B.StreamCfgC.path_stats.offset, B.StreamCfgC.path_stats_cap.offset]
    assert got == want


def test_file_tier_argument_errors(tmp_path):
    hp = B.HParams()
    T = 1024
    n = 3000
    state_bytes = B.mlpo_state_floats(n, T) * 4
    path = tmp_path / "state.bin"
    path.write_bytes(bytes(4096 + state_bytes))
    fd = os.open(str(path), os.O_RDWR)
    try:
        filesg = B.SubgroupC(None, None, None, FAKE, FAKE + (1 << 20), n, B.TIER_FILE, T)
        need = B.mlpo_stream_bounce_bytes([filesg], 2, 0)
        assert need == 2 * state_bytes and state_bytes % 4096 == 0
        assert B.mlpo_stream_bounce_bytes([filesg], 3, 1024) == 3 * 3 * 1024 * 4
        assert B.mlpo_stream_bounce_bytes([sg(n=1000, tier=1)], 3, 0) == 0

        def cfg(**kw):
            args = dict(files=[(fd, 4096)], bounce=FAKE_PAGE, bounce_bytes=need, file_slots=2)
            args.update(kw)
            return B.direct_cfg(None, None, 8, **args)

        expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [filesg], hp, 1)                            # needs the pipeline
        staged = B.stream_cfg(2, FAKE, 1 << 30, None, None, None, 0)
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, staged)     # needs direct mode
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, B.direct_cfg(None, None, 8))
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(file_slots=0))
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(file_slots=B.MAX_SLOTS + 1))
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(bounce=0))
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(bounce=FAKE_PAGE + 512))
        expect(B.MLPO_ENOMEM, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(bounce_bytes=need - 1))
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(files=[(fd, 100)]))   # offset
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(files=[(fd, 8192)]))  # too short
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(files=[(10_000, 0)]))  # bad fd
        r, w = os.pipe()
        try:
            expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(files=[(r, 0)]))  # a pipe
        finally:
            os.close(r)
            os.close(w)
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(chunk_elems=1536))     # not k * T
        with_ptr = B.SubgroupC(FAKE, FAKE + 4 * T, FAKE + 8 * T, FAKE, FAKE + (1 << 20), n, B.TIER_FILE, T)
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [with_ptr], None, hp, 1, None, cfg())
        planar = B.SubgroupC(None, None, None, FAKE, FAKE + (1 << 20), n, B.TIER_FILE, 0)
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [planar], None, hp, 1, None, cfg())
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(file_threads=-1))
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [filesg], None, hp, 1, None, cfg(file_threads=17))
    finally:
        os.close(fd)


def test_half_format_errors():
    hp = B.HParams()
    bad = hp.c()
    bad.l2_mode = 2
    assert B.lib().mlpo_adamw_step(None, 0, C.byref(bad), 1, None, None) == B.MLPO_EINVAL
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(half_format=2)], hp, 1)
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(), sg(half_format=B.HALF_FP16)], hp, 1)     # mixed formats
    # lead: a multiple of 4 below 1024, tiled layout, HBM tier
    tiled = dict(p=FAKE_PAGE, m=FAKE_PAGE + 4 * 1024, v=FAKE_PAGE + 8 * 1024, tile_elems=1024)
    for bad_lead in (1, 2, -4, 1024, 4096):
        expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(lead=bad_lead, **tiled)], hp, 1)
    expect(B.MLPO_EINVAL, B.mlpo_adamw_step, [sg(lead=8)], hp, 1)                               # planar
    expect(B.MLPO_EINVAL, B.mlpo_stream_update, [sg(lead=8, tier=B.TIER_HOST, **tiled)], None, hp, 1, None,
           B.direct_cfg(None, None, 8))                                                         # not HBM-tier
    expect(B.MLPO_EINVAL, B.mlpo_state_pack, FAKE, FAKE, FAKE, 10, 1024, FAKE, lead=2)
    expect(B.MLPO_EINVAL, B.mlpo_state_unpack, FAKE, 10, 1024, FAKE, FAKE, FAKE, lead=1024)
    expect(B.MLPO_EINVAL, B.mlpo_grad_unscale_norm, [sg(half_format=-1)], 1.0, 0.0, FAKE, B.mlpo_norm_workspace_bytes(),
           FAKE)
    expect(B.MLPO_EINVAL, B.mlpo_grad_accumulate, FAKE, FAKE + 4096, 16, half=2)


def test_flush_target_argument_errors(tmp_path):
    hp = B.HParams()
    T, n = 1024, 3000
    floats = B.mlpo_state_floats(n, T)
    path = tmp_path / "state.bin"
    path.write_bytes(bytes(2 * floats * 4))
    fd = os.open(str(path), os.O_RDWR)
    try:
        hostsg = B.tiled_subgroup(FAKE_PAGE, FAKE, FAKE + (1 << 20), n=n, tier=B.TIER_HOST, tile_elems=T)
        other = FAKE_PAGE + (1 << 30)

        def cfg(target, **kw):
            args = dict(bounce=FAKE_PAGE + (2 << 30), bounce_bytes=1 << 30, file_slots=2, flush_to=[target])
            args.update(kw)
            return B.direct_cfg(None, None, 8, **args)

        # to a file: the bounce buffers are needed even though nothing is file-tier yet
        assert B.mlpo_stream_bounce_bytes([hostsg], 2, 0) == 0
        assert B.mlpo_stream_bounce_bytes([hostsg], 2, 0, flush_to=[(fd, 0)]) == 2 * floats * 4
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hostsg], None, hp, 1, None, cfg((fd, 0), bounce=0))
        expect(B.MLPO_ENOMEM, B.mlpo_stream_update, [hostsg], None, hp, 1, None, cfg((fd, 0), bounce_bytes=4096))
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hostsg], None, hp, 1, None, cfg((fd, 100)))        # offset
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hostsg], None, hp, 1, None, cfg((fd, 2 * floats * 4)))  # too short
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hostsg], None, hp, 1, None, cfg(other + 64))       # alignment
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hostsg], None, hp, 1, None, cfg(FAKE_PAGE + 256))  # overlaps
        bad = cfg(other)
        bad._flush[0].tier = 7
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hostsg], None, hp, 1, None, bad)
        bad = cfg(other)
        bad._flush[0].reserved = 1
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hostsg], None, hp, 1, None, bad)
        planar = sg(n=n, tier=B.TIER_HOST)
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [planar], None, hp, 1, None, cfg(other))            # planar layout
        hbm = B.tiled_subgroup(FAKE_PAGE, FAKE, FAKE + (1 << 20), n=n, tier=B.TIER_HBM, tile_elems=T)
        to_hbm = B.FlushTargetC(B.TIER_HBM, 0, other, B.FileExtentC(-1, 0, 0))
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hbm], None, hp, 1, None, cfg(to_hbm))              # HBM to HBM
        host_g = B.tiled_subgroup(FAKE_PAGE, FAKE, FAKE + (1 << 20), n=n, tier=B.TIER_HOST_GRADS, tile_elems=T)
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [host_g], None, hp, 1, None, cfg(to_hbm))           # gradients stay
        hbm_planar = sg(n=n, tier=B.TIER_HBM)
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hbm_planar], None, hp, 1, None, cfg(other))        # planar layout
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hbm], None, hp, 1, None, cfg(other, chunk_elems=T + 4))
        staged = B.stream_cfg(2, FAKE, 1 << 30, None, None, None, 0)
        staged._flush = B.flush_targets([other])
        staged.flush_to = staged._flush
        expect(B.MLPO_EINVAL, B.mlpo_stream_update, [hostsg], None, hp, 1, None, staged)                # staged mode
    finally:
        os.close(fd)
