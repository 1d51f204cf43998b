"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; GPU sanitizers are not available here): the
oracle against its pins, and the library's host-side argument checks, arena and tables against the C-ABI tests that need no
GPU.  Each side runs in a process of its own with its compiler's sanitizer runtime preloaded; any report fails the run."""
from paper_2310_12403_amd import build


def test_host_code_is_clean_under_asan_and_ubsan():
    assert build.sanitize_check(verbose=False)
