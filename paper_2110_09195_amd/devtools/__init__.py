"""Developer tools: summarisers of rocprofv3 output and an instrumented build of the stack kernel (not imported by
the library, the tests or bench.py)."""
