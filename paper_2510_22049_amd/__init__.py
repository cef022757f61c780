"""MI355X-native hot path of VISTA (virtual-seed history summarization and
candidate target attention).  The compute lives in ``libvista.so`` (hand-written
HIP behind a C ABI); ``binding`` marshals arguments to it and ``inputs`` draws
the seeded synthetic workloads.  Nothing here computes on the CPU."""

__all__ = ["binding", "inputs", "build"]
