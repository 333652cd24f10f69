"""The hand-scheduled (inline-asm) loads of the kernels must never have their destination
registers copied, spilled or reused while in flight.  Compiles the kernels to assembly (no GPU
needed) and scans them; also checks the scanner itself on two hand-written snippets."""
import isa_check


def test_scanner_flags_a_copy_of_an_in_flight_register():
    bad = isa_check.check_kernel([
        "global_load_dwordx4 v[10:13], v[0:1], off",
        "v_mov_b32_e32 v20, v11",
        "s_waitcnt vmcnt(0)",
        "v_mov_b32_e32 v21, v12",
        "s_endpgm",
    ])
    assert [b[0] for b in bad] == [2]


def test_scanner_accepts_ordered_waits():
    bad = isa_check.check_kernel([
        "global_load_dwordx4 v[10:13], v[0:1], off",
        "global_load_dwordx4 v[14:17], v[0:1], off offset:1024",
        "s_waitcnt vmcnt(1)",
        "v_mfma_f32_32x32x2_f32 v[32:47], v10, v4, v[32:47]",
        "s_waitcnt vmcnt(0)",
        "v_mfma_f32_32x32x2_f32 v[32:47], v14, v4, v[32:47]",
        "s_endpgm",
    ])
    assert bad == []


def test_scanner_counts_stores_in_vmcnt():
    # a compiler-placed wait behind two stores: vmcnt(2) retires the load
    ok = isa_check.check_kernel([
        "global_load_dword v10, v[0:1], off",
        "global_store_dword v[2:3], v5, off",
        "global_store_dword v[2:3], v6, off offset:4",
        "s_waitcnt vmcnt(2)",
        "v_add_f32_e32 v7, v10, v10",
        "s_endpgm",
    ])
    assert ok == []
    bad = isa_check.check_kernel([
        "global_load_dword v10, v[0:1], off",
        "global_store_dword v[2:3], v5, off",
        "s_waitcnt vmcnt(2)",
        "v_add_f32_e32 v7, v10, v10",
        "s_endpgm",
    ])
    assert [b[0] for b in bad] == [4]


def test_compiled_kernels_have_no_in_flight_register_hazard():
    res = isa_check.check_all(isa_check.compile_to_asm())
    assert len(res) >= 3  # STFT, Mel and CQT kernels
    for name, bad in res.items():
        assert bad == [], (name, bad[:5])
