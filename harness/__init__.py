"""Seeded synthetic inputs of the named workloads (synth) and the data movement that primes a device cache with
them (workloads).  Shared by the tests, bench.py and the smoke check; holds none of the method's arithmetic, and
neither the library binding nor the oracle depends on it for anything but inputs."""
