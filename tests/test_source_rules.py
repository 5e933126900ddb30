"""Rules the kernel sources are held to, checked on the text (no GPU needed).

* Inline assembly may hold no instruction whose register operands the compiler has to guard: on
  gfx950 the wait states between a matrix instruction and a vector instruction that reads its
  result are inserted by the compiler, for the instructions it emits itself.  Allowed are empty
  templates (register constraints only) and the direct-to-LDS request with its M0 set-up.
* No packed fp32 arithmetic written by hand, and the build switches the compiler's own off.
"""
import pathlib
import re

ROOT = pathlib.Path(__file__).resolve().parents[1]
CSRC = ROOT / "paper_2603_13420_amd" / "csrc"
SOURCES = sorted(p for p in CSRC.iterdir() if p.suffix in (".hip", ".hpp", ".h", ".cpp"))


def asm_templates(text):
    """The string literal(s) that open every asm(...) / asm volatile(...) statement."""
    for m in re.finditer(r"\basm\s*(?:volatile\s*)?\(\s*((?:\"(?:[^\"\\]|\\.)*\"\s*)+)", text):
        yield "".join(re.findall(r"\"((?:[^\"\\]|\\.)*)\"", m.group(1)))


def test_sources_exist():
    assert len(SOURCES) >= 6


def test_inline_assembly_is_constraints_only_or_the_lds_request():
    for p in SOURCES:
        for t in asm_templates(p.read_text()):
            ok = t == "" or ("global_load_lds_dwordx4" in t and "s_mov_b32 m0" in t)
            assert ok, f"{p.name}: inline instruction(s) {t!r}: use a compiler intrinsic instead"


def test_an_asm_statement_that_writes_m0_says_so_in_its_clobber_list():
    """The compiler may keep a value of its own in M0 across an asm statement unless told otherwise."""
    for p in SOURCES:
        text = p.read_text()
        for m in re.finditer(r"\basm\s*(?:volatile\s*)?\(", text):
            depth, i = 1, m.end()
            while depth and i < len(text):      # the whole statement, up to its closing parenthesis
                depth += {"(": 1, ")": -1}.get(text[i], 0)
                i += 1
            stmt = text[m.start():i]
            if re.search(r"\bm0\s*,", "".join(re.findall(r"\"((?:[^\"\\]|\\.)*)\"", stmt.split(":")[0]))):
                clobbers = stmt.rsplit(":", 1)[1]
                assert '"m0"' in clobbers, f"{p.name}: asm statement writes m0 without declaring the clobber"


def test_no_packed_fp32_by_hand_and_the_flag_is_set():
    for p in SOURCES:
        text = p.read_text()
        for word in ("v_pk_add_f32", "v_pk_mul_f32", "v_pk_fma_f32"):
            assert word not in text, f"{p.name}: {word}"
    build = (ROOT / "paper_2603_13420_amd" / "build.py").read_text()
    assert "-packed-fp32-ops" in build and "-target-feature" in build
