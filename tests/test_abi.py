"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes the state as Table 1 of the paper says, and rejects bad arguments before
anything is launched."""
import ctypes as C
import os
import re

import pytest

import paper_2412_05270_amd as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**kw):
    base = dict(rank=4, mode=A.APOLLO_CHANNEL, seed=1, beta1=0.9, beta2=0.999, eps=1e-8, scale=1.0,
                weight_decay=0.0, nl_gamma=1.01, refresh_interval=200, bias_correction=1,
                side=A.APOLLO_SIDE_AUTO, weight_dtype=A.APOLLO_F32, state_dtype=A.APOLLO_F32, projection=A.APOLLO_PROJ_RANDOM,
                weight_rounding=A.APOLLO_ROUND_NEAREST, schedule=A.APOLLO_SCHEDULE_SERIAL)
    base.update(kw)
    return A.ApolloConfig(**base)


def test_library_exports_every_declared_symbol():
    lib = A.load_library()
    header = open(os.path.join(ROOT, "include", "apollo.h")).read()
    names = set(re.findall(r"\b(apollo_[a-z_]+)\s*\(", header))
    assert {"apollo_init", "apollo_step", "apollo_state_bytes", "apollo_workspace_bytes", "apollo_destroy",
            "apollo_debug_fill_projection", "apollo_debug_get", "apollo_state_offsets", "apollo_last_error",
            "apollo_debug_philox", "apollo_debug_gauss_parts", "apollo_debug_copy", "apollo_debug_path", "apollo_profile_enable",
            "apollo_profile_read", "apollo_step_noalloc", "apollo_step_prepare", "apollo_step_launch", "apollo_adamw_state_bytes", "apollo_adamw_state_offsets",
            "apollo_adamw_workspace_bytes", "apollo_adamw_init", "apollo_adamw_step", "apollo_adamw_last_error",
            "apollo_adamw_destroy"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_struct_sizes_match_the_header_layout():
    assert C.sizeof(A.ApolloShape) == 24
    assert C.sizeof(A.ApolloConfig) == 72
    assert C.sizeof(A.ApolloTensor) == 24
    assert C.sizeof(A.ApolloFlatShape) == 16
    assert C.sizeof(A.ApolloAdamwConfig) == 24


def test_header_is_plain_c_and_agrees_with_the_binding(tmp_path):
    """The header compiles as C99 on its own; the sizes, field offsets and constants a C caller gets
    are the ones the ctypes binding uses."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "probe.c"
    src.write_text("""
#include <stdio.h>
#include <stddef.h>
#include "apollo.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu\\n", sizeof(apollo_shape_t), sizeof(apollo_config_t), sizeof(apollo_tensor_t),
         sizeof(apollo_flat_shape_t), sizeof(apollo_adamw_config_t));
  printf("%zu %zu %zu %zu %zu %zu %zu\\n", offsetof(apollo_config_t, seed), offsetof(apollo_config_t, beta1),
         offsetof(apollo_config_t, refresh_interval), offsetof(apollo_config_t, weight_dtype),
         offsetof(apollo_config_t, schedule), offsetof(apollo_tensor_t, w_meta), offsetof(apollo_shape_t, grad_dtype));
  printf("%d %d %d %d %d %d %d %d %d %d\\n", APOLLO_BF16, APOLLO_Q8, APOLLO_TENSOR, APOLLO_SIDE_RIGHT, APOLLO_PROJ_IDENTITY,
         APOLLO_ROUND_STOCHASTIC, APOLLO_SCHEDULE_OVERLAP, APOLLO_DBG_COLSQ, APOLLO_EUNSUPPORTED, APOLLO_ESTATE);
  return 0;
}
""")
    exe = tmp_path / "probe"
    subprocess.run([cc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    sizes = [int(x) for x in out[0].split()]
    assert sizes == [C.sizeof(A.ApolloShape), C.sizeof(A.ApolloConfig), C.sizeof(A.ApolloTensor),
                     C.sizeof(A.ApolloFlatShape), C.sizeof(A.ApolloAdamwConfig)]
    offs = [int(x) for x in out[1].split()]
    assert offs == [A.ApolloConfig.seed.offset, A.ApolloConfig.beta1.offset, A.ApolloConfig.refresh_interval.offset,
                    A.ApolloConfig.weight_dtype.offset, A.ApolloConfig.schedule.offset, A.ApolloTensor.w_meta.offset,
                    A.ApolloShape.grad_dtype.offset]
    consts = [int(x) for x in out[2].split()]
    assert consts == [A.APOLLO_BF16, A.APOLLO_Q8, A.APOLLO_TENSOR, A.APOLLO_SIDE_RIGHT, A.APOLLO_PROJ_IDENTITY,
                      A.APOLLO_ROUND_STOCHASTIC, A.APOLLO_SCHEDULE_OVERLAP, A.APOLLO_DBG_COLSQ, A.APOLLO_EUNSUPPORTED,
                      A.APOLLO_ESTATE]


def test_state_bytes_follow_table_1():
    # 2 n r moments + 1 norm per tensor, n the larger dimension; blocks 256-byte aligned
    shapes = [(8, 20, A.APOLLO_F32), (20, 8, A.APOLLO_BF16)]
    cfg = _cfg(rank=4)
    per = (2 * 4 * 20 + 1) * 4
    per_aligned = (per + 255) // 256 * 256
    assert A.apollo_state_bytes(cfg, shapes) == 2 * per_aligned
    rc, m, v, nm = A.apollo_state_offsets(cfg, shapes, 1)
    assert (rc, m, v, nm) == (0, per_aligned, per_aligned + 4 * 20 * 4, per_aligned + 2 * 4 * 20 * 4)
    # LLaMA-7B at r = 256: 809 500 672 moment elements (the paper's 1.6G in bf16)
    llama = ([(4096, 4096, 1)] * 4 + [(11008, 4096, 1)] * 2 + [(4096, 11008, 1)]) * 32
    sb = A.apollo_state_bytes(_cfg(rank=256), llama)
    assert sb >= 4 * (809_500_672 + 224) and sb < 4 * (809_500_672 + 224) + 256 * 224
    # forcing the side changes which dimension carries the channels
    assert A.apollo_state_bytes(_cfg(rank=4, side=A.APOLLO_SIDE_RIGHT), [(8, 20, 0)]) == \
        ((2 * 4 * 8 + 1) * 4 + 255) // 256 * 256


@pytest.mark.parametrize("kw,shapes,code", [
    (dict(rank=0), [(8, 8, 0)], A.APOLLO_EINVAL),
    (dict(rank=9), [(8, 16, 0)], A.APOLLO_EINVAL),            # rank above the projected dimension
    (dict(rank=9, side=A.APOLLO_SIDE_RIGHT), [(16, 8, 0)], A.APOLLO_EINVAL),
    (dict(refresh_interval=0), [(8, 8, 0)], A.APOLLO_EINVAL),
    (dict(mode=7), [(8, 8, 0)], A.APOLLO_EINVAL),
    (dict(side=5), [(8, 8, 0)], A.APOLLO_EINVAL),
    (dict(beta1=1.0), [(8, 8, 0)], A.APOLLO_EINVAL),
    (dict(eps=-1.0), [(8, 8, 0)], A.APOLLO_EINVAL),
    (dict(), [(0, 8, 0)], A.APOLLO_EINVAL),
    (dict(), [(8, 8, 3)], A.APOLLO_EUNSUPPORTED),             # fp16 / fp8 gradients are not supported
    (dict(), [(8, (1 << 20) + 1, 0)], A.APOLLO_EUNSUPPORTED),
    (dict(), [], A.APOLLO_EINVAL),
])
def test_bad_arguments_are_rejected_before_any_launch(kw, shapes, code):
    cfg = _cfg(**kw)
    assert A.apollo_state_bytes(cfg, shapes) == 0
    assert A.apollo_workspace_bytes(cfg, shapes) == 0
    rc, h = A.apollo_init(cfg, shapes, 256, 1 << 30, 512, 1 << 30)      # fake aligned pointers: never touched
    assert rc == code and h is None
    assert A.apollo_last_error() != ""


def test_init_rejects_small_or_misaligned_buffers_without_touching_them():
    cfg = _cfg()
    shapes = [(8, 8, 0)]
    sb, wb = A.apollo_state_bytes(cfg, shapes), A.apollo_workspace_bytes(cfg, shapes)
    assert sb > 0 and wb > 0
    assert A.apollo_init(cfg, shapes, 256, sb - 1, 512, wb)[0] == A.APOLLO_ESTATE
    assert A.apollo_init(cfg, shapes, 256, sb, 512, wb - 1)[0] == A.APOLLO_ESTATE
    assert A.apollo_init(cfg, shapes, 264, sb, 512, wb)[0] == A.APOLLO_ESTATE
    assert A.apollo_init(cfg, shapes, None, sb, 512, wb)[0] == A.APOLLO_EINVAL
    assert A.apollo_init(None, shapes, 256, sb, 512, wb)[0] == A.APOLLO_EINVAL


def test_storage_types_are_validated_and_size_the_state():
    shapes = [(8, 20, A.APOLLO_F32)]
    per32 = ((2 * 4 * 20 * 4 + 4) + 255) // 256 * 256
    per16 = ((2 * 4 * 20 * 2 + 4) + 255) // 256 * 256
    assert A.apollo_state_bytes(_cfg(rank=4), shapes) == per32
    assert A.apollo_state_bytes(_cfg(rank=4, state_dtype=A.APOLLO_BF16), shapes) == per16
    assert A.apollo_state_bytes(_cfg(rank=4, weight_dtype=A.APOLLO_BF16), shapes) == per32
    cfg = _cfg(rank=4, state_dtype=A.APOLLO_BF16)
    assert A.apollo_state_offsets(cfg, shapes, 0) == (0, 0, 4 * 20 * 2, 2 * 4 * 20 * 2)
    assert A.apollo_state_bytes(_cfg(state_dtype=2), shapes) == 0
    assert A.apollo_state_bytes(_cfg(weight_dtype=-1), shapes) == 0
    assert "dtype" in A.apollo_last_error()


def test_identity_projection_sizes_full_rank_state_and_ignores_the_rank():
    shapes = [(8, 20, A.APOLLO_F32), (20, 8, A.APOLLO_BF16)]
    per = ((2 * 8 * 20 * 4 + 4) + 255) // 256 * 256
    for rank in (0, 4, 1000):
        assert A.apollo_state_bytes(_cfg(rank=rank, projection=A.APOLLO_PROJ_IDENTITY), shapes) == 2 * per
    assert A.apollo_state_bytes(_cfg(projection=2), shapes) == 0
    assert A.apollo_state_bytes(_cfg(rank=0), shapes) == 0


def test_unknown_schedule_and_rounding_are_rejected():
    assert A.apollo_state_bytes(_cfg(schedule=3), [(8, 8, 0)]) == 0
    assert A.apollo_state_bytes(_cfg(schedule=A.APOLLO_SCHEDULE_CHUNKED), [(8, 8, 0)]) > 0
    assert A.apollo_state_bytes(_cfg(weight_rounding=5), [(8, 8, 0)]) == 0
    assert A.apollo_state_bytes(_cfg(schedule=A.APOLLO_SCHEDULE_OVERLAP), [(8, 8, 0)]) > 0


def test_null_handle_calls_fail_cleanly():
    assert A.apollo_step(None, [(16, 32)], 1, 0.1) == A.APOLLO_EINVAL
    assert A.apollo_step_prepare(None, 1, 0.1) == A.APOLLO_EINVAL
    assert A.apollo_step_launch(None, None) == A.APOLLO_EINVAL
    assert A.apollo_debug_get(None, 0, A.APOLLO_DBG_M, 16, 4) == A.APOLLO_EINVAL
    assert A.apollo_debug_fill_projection(None, 0, 1, 16, A.APOLLO_F32) == A.APOLLO_EINVAL
    assert A.apollo_debug_gauss_parts(1 << 24, 1, 16, 16, 16) == A.APOLLO_EINVAL
    A.apollo_destroy(None)


def test_noalloc_step_rejects_oversized_and_bad_requests_before_any_launch():
    """Every check of apollo_step_noalloc comes before its first GPU call: too many tensors, a list whose
    scratch exceeds the static array, and the argument errors of apollo_init / apollo_step."""
    cfg = _cfg(rank=4)
    one = [(8, 8, 0)]
    ptrs = [(4096, 8192)]                                    # fake aligned pointers: never touched
    sb = A.apollo_state_bytes(cfg, one)
    many = one * (A.APOLLO_NOALLOC_MAX_TENSORS + 1)
    assert A.apollo_step_noalloc(cfg, many, ptrs * len(many), 256, 1 << 30, 1, 1, 0.1) == A.APOLLO_EUNSUPPORTED
    assert "at most 64" in A.apollo_last_error()
    # four LLaMA-7B matrices at rank 1024 need more scratch (their P alone) than the static array holds
    big = [(4096, 11008, A.APOLLO_BF16)] * 4
    need = A.apollo_workspace_bytes(_cfg(rank=1024), big)
    assert need > A.APOLLO_NOALLOC_SCRATCH_BYTES
    assert A.apollo_step_noalloc(_cfg(rank=1024), big, ptrs * 4, 256, 1 << 40, 1, 1, 0.1) == A.APOLLO_EUNSUPPORTED
    msg = A.apollo_last_error()
    assert str(need) in msg and str(A.APOLLO_NOALLOC_SCRATCH_BYTES) in msg
    assert A.apollo_step_noalloc(cfg, one, ptrs, 256, sb - 1, 1, 1, 0.1) == A.APOLLO_ESTATE
    assert A.apollo_step_noalloc(cfg, one, ptrs, 264, sb, 1, 1, 0.1) == A.APOLLO_ESTATE
    assert A.apollo_step_noalloc(cfg, one, ptrs, None, sb, 1, 1, 0.1) == A.APOLLO_EINVAL
    assert A.apollo_step_noalloc(cfg, one, None, 256, sb, 1, 1, 0.1) == A.APOLLO_EINVAL
    assert A.apollo_step_noalloc(cfg, one, ptrs, 256, sb, 1, 0, 0.1) == A.APOLLO_EINVAL            # step < 1
    assert A.apollo_step_noalloc(cfg, one, ptrs, 256, sb, 1, 1, float("nan")) == A.APOLLO_EINVAL
    assert A.apollo_step_noalloc(cfg, one, [(4100, 8192)], 256, sb, 1, 1, 0.1) == A.APOLLO_EINVAL  # misaligned W
    assert A.apollo_step_noalloc(_cfg(rank=0), one, ptrs, 256, sb, 1, 1, 0.1) == A.APOLLO_EINVAL
    assert A.apollo_step_noalloc(None, one, ptrs, 256, sb, 1, 1, 0.1) == A.APOLLO_EINVAL


# ------------------------------------------------------------------ element-wise AdamW entry points
def _acfg(**kw):
    base = dict(beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, bias_correction=1, reserved=0)
    base.update(kw)
    return A.ApolloAdamwConfig(**base)


def test_adamw_state_layout():
    # per tensor M then V, each starting on a 256-byte boundary
    shapes = [(100, A.APOLLO_F32), (5, A.APOLLO_BF16), (64, A.APOLLO_BF16)]
    assert A.apollo_adamw_state_bytes(shapes) == 512 + 512 + 256 + 256 + 256 + 256
    assert A.apollo_adamw_state_offsets(shapes, 0) == (0, 0, 512)
    assert A.apollo_adamw_state_offsets(shapes, 1) == (0, 1024, 1280)
    assert A.apollo_adamw_state_offsets(shapes, 2) == (0, 1536, 1792)
    assert A.apollo_adamw_state_offsets(shapes, 3)[0] == A.APOLLO_EINVAL
    # workspace: descriptor table (48 bytes per tensor) and one table entry per block of 1024 elements
    assert A.apollo_adamw_workspace_bytes([(1024, 0)]) == 256 + 256
    assert A.apollo_adamw_workspace_bytes([(1025, 0)] * 7) == 512 + 256
    assert A.apollo_adamw_workspace_bytes([(1024 * 200, 1)]) == 256 + 1024
    # bfloat16 storage halves a tensor's state
    mixed = [(100, A.APOLLO_F32, A.APOLLO_BF16), (100, A.APOLLO_F32, A.APOLLO_F32)]
    assert A.apollo_adamw_state_bytes(mixed) == 256 + 256 + 512 + 512
    assert A.apollo_adamw_state_offsets(mixed, 0) == (0, 0, 256)
    assert A.apollo_adamw_state_offsets(mixed, 1) == (0, 512, 1024)
    assert A.apollo_adamw_state_bytes([(100, A.APOLLO_F32, 5)]) == 0 and "storage" in A.apollo_adamw_last_error()


def test_adamw_bad_arguments_are_rejected_before_any_launch():
    assert A.apollo_adamw_state_bytes([]) == 0
    assert A.apollo_adamw_state_bytes([(0, 0)]) == 0
    assert A.apollo_adamw_state_bytes([(8, 7)]) == 0
    assert "dtype" in A.apollo_adamw_last_error()
    assert A.apollo_adamw_state_bytes([((1 << 40) + 1, 0)]) == 0
    shapes = [(1000, 0)]
    sb, wb = A.apollo_adamw_state_bytes(shapes), A.apollo_adamw_workspace_bytes(shapes)
    for bad in (dict(beta1=1.0), dict(beta2=-0.1), dict(eps=-1.0), dict(weight_decay=float("inf")),
                dict(bias_correction=2)):
        assert A.apollo_adamw_init(_acfg(**bad), shapes, 256, sb, 512, wb)[0] == A.APOLLO_EINVAL
    assert A.apollo_adamw_init(_acfg(), shapes, 256, sb - 1, 512, wb)[0] == A.APOLLO_ESTATE
    assert A.apollo_adamw_init(_acfg(), shapes, 256, sb, 512, wb - 1)[0] == A.APOLLO_ESTATE
    assert A.apollo_adamw_init(_acfg(), shapes, 260, sb, 512, wb)[0] == A.APOLLO_ESTATE
    assert A.apollo_adamw_init(_acfg(), shapes, None, sb, 512, wb)[0] == A.APOLLO_EINVAL
    assert A.apollo_adamw_init(None, shapes, 256, sb, 512, wb)[0] == A.APOLLO_EINVAL
    assert A.apollo_adamw_step(None, [(16, 32)], 1, 0.1) == A.APOLLO_EINVAL
    A.apollo_adamw_destroy(None)


def test_the_chunked_schedule_keeps_scratch_for_one_chunk_of_projections():
    """APOLLO_SCHEDULE_CHUNKED: the workspace holds the P of at most 128 MiB worth of tensors (of one
    shape group at a time) instead of every tensor's: the LLaMA-7B matrices at rank 256 need 0.48 GB with
    the default schedule, a quarter of that with this one; rank 1 has no scratch copy of P either way;
    the state does not depend on the schedule."""
    shapes = []
    for _ in range(32):
        shapes += [(4096, 4096, A.APOLLO_BF16)] * 4 + [(11008, 4096, A.APOLLO_BF16)] * 2 + [(4096, 11008, A.APOLLO_BF16)]
    serial = A.apollo_workspace_bytes(_cfg(rank=256), shapes)
    chunked = A.apollo_workspace_bytes(_cfg(rank=256, schedule=A.APOLLO_SCHEDULE_CHUNKED), shapes)
    p_all = 224 * 256 * 4096 * 2
    assert serial - chunked == p_all - (128 << 20)
    assert A.apollo_state_bytes(_cfg(rank=256), shapes) == A.apollo_state_bytes(_cfg(rank=256, schedule=A.APOLLO_SCHEDULE_CHUNKED), shapes)
    mini = dict(rank=1, mode=A.APOLLO_TENSOR)
    assert A.apollo_workspace_bytes(_cfg(**mini), shapes) == A.apollo_workspace_bytes(_cfg(schedule=A.APOLLO_SCHEDULE_CHUNKED, **mini), shapes)
