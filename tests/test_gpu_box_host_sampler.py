"""The multi-threaded host sampler (Tab. I, "Sampling Device = CPU") on the machine whose GPU
runs the other tests: it picks its vector code from the host CPU at run time, so the form that
bench.py's cpu_sampler leg times has to be compared with the oracle there, not only on the
machine that builds the library.  No GPU call is made; the marker only places the run."""
import pytest

import paper_2511_07421_amd as a3
import test_cpu_sampler as host

pytestmark = pytest.mark.gpu


def test_vector_forms_agree_on_this_machine():
    differ, forms = a3.check_vector_forms()
    print(f"[case] vector forms of the draws on this CPU: {forms}", flush=True)
    assert differ == 0


@pytest.mark.parametrize("form", [0, 1, 2, 3])
def test_host_sampler_matches_oracle_in_the_picked_and_in_every_forced_form(form):
    """0: the form the sampler picks by itself here; 1, 2, 3: scalar, AVX2, AVX-512 forced"""
    host.test_cpu_sampler_matches_oracle_in_every_vector_form(form)


@pytest.mark.parametrize("name", ["mini_copurchase", "mini_citation"])
def test_host_sampler_matches_oracle_on_both_id_widths(name):
    host.test_cpu_sampler_matches_oracle(name)
